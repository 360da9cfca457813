"""GPU parity for the features used together: every layer of a model, shared prefix pages, token-level page
masks, explicit bitmaps, LoRA adapters, positions recorded by embed_txt, forward + distribution in one call."""
import numpy as np
import pytest

import workloads as W
from oracle import pie_oracle as O
from helpers import check_topk, clone_batch, deep_oracle_pools
from gpu_helpers import assert_close, dec
from test_gpu_adapter import ALL, make_ctx

pytestmark = pytest.mark.gpu


def hide(a0, a1):
    def f(n_new, L, rng):
        m = W.causal_bitmap(n_new, L)
        m[:, a0:a1] = False
        return m
    return f


@pytest.mark.parametrize("head_dim,n_q,n_kv", [(64, 4, 2), (128, 8, 2)])
def test_everything_together(head_dim, n_q, n_kv):
    m = W.ModelDesc(hidden=128, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=head_dim, mlp_dim=256, vocab=512, page_size=16,
                    rms_eps=1e-5, rope_theta=1e4, n_layers=3)
    P = 16
    reqs = [W.RequestSpec(1, 4 * P + 3, prefix_group=0, prefix_len=4 * P),
            W.RequestSpec(1, 4 * P + 11, prefix_group=0, prefix_len=4 * P, mask=hide(P, 2 * P + 5)),
            W.RequestSpec(1, 4 * P + 30, prefix_group=0, prefix_len=4 * P, in_place=True),
            W.RequestSpec(2, 5 * P, prefix_group=0, prefix_len=4 * P, mask=W.causal_bitmap),
            W.RequestSpec(37, 4 * P, prefix_group=0, prefix_len=4 * P),       # prefill over the shared prefix
            W.RequestSpec(1, 90), W.RequestSpec(20, 0, store_all_rows=False)]
    dw = W.build_deep_workload("combined", m, reqs, n_kv_pages=96, seed=7000 + head_dim, std=0.05,
                               resid_std=0.05 / np.sqrt(6.0), top_k=12)
    w, b = dw.base, dw.base.batch
    adapters = {0: W.make_adapter(m, 7000, 0, rank=8, projections=ALL, scale=1.0, std=0.05),
                1: W.make_adapter(m, 7000, 1, rank=3, projections=("wq", "wk", "wv", "wo"), scale=2.0, std=0.05)}
    adapter_ids = np.array([0, 1, -1, 0, 1, -1, 0], np.int32)
    rng = np.random.default_rng(7)
    pages = np.unique(b.page_ids)[::3].astype(np.int32)   # includes shared prefix pages
    bits = rng.integers(0, 1 << 16, size=len(pages)).astype(np.uint32)
    bits[1] = 0

    ctx = make_ctx(dw, adapters, 8)
    ctx.embed_txt(dw.token_ids, b.positions, b.in_embed_ids)
    ctx.mask_kvpage(pages, bits)
    bb = clone_batch(b, positions=None, adapter_ids=adapter_ids)
    pb = ctx.batch_create(bb)
    ctx.forward_all(pb)
    ctx.synchronize()
    stored = np.nonzero(b.out_embed_ids >= 0)[0]
    y_bits = ctx.embed_read(b.out_embed_ids[stored])

    kvs, emb = deep_oracle_pools(dw)
    O.embed_txt(dw.table_bits, dw.token_ids, b.positions, emb, b.in_embed_ids)
    O.mask_kvpage(kvs, pages, bits)
    res = O.forward_model(m, dw.layers, kvs, emb, b, round_intermediates=True, adapters=adapters, adapter_ids=adapter_ids)
    assert_close(dec(y_bits), res[-1].y[stored], f"everything together D{head_dim}")
    work = pb.work()
    assert work["kv_bytes_requested"] < work["kv_bytes_decode"]  # the shared prefix was grouped
