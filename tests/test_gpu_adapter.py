"""GPU parity (through the C ABI) for LoRA adapters (`forward_with_adapter`): per-request low-rank updates of
the layer's projections, against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

import workloads as W
from oracle import pie_oracle as O
from helpers import clone_batch, deep_oracle_pools
from gpu_helpers import appended_positions, assert_bf16_close, assert_close, dec

pytestmark = pytest.mark.gpu

ALL = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")


def make_ctx(dw, adapters, max_rank):
    from paper_2510_24051_amd import Pie
    w, b = dw.base, dw.base.batch
    ctx = Pie(w.model, w.n_kv_pages, w.n_embeds, max_batch_tokens=b.n_tokens, max_batch_requests=b.n_requests,
              max_top_k=16, max_dist_rows=0, n_layers=w.model.n_layers, max_adapters=max(adapters) + 1 if adapters else 0,
              max_lora_rank=max_rank)
    for l, lw in enumerate(dw.layers):
        ctx.load_layer(l, lw)
    ctx.load_embedding(dw.table_bits)
    for l, pr in enumerate(dw.priors):
        if len(pr.page_ids):
            ctx.kv_write(l, pr.page_ids, pr.slots, pr.k_bits, pr.v_bits)
    for a, layers in adapters.items():
        ctx.load_adapter(a, layers)
    return ctx


def compare(dw, adapters, adapter_ids, what, max_rank=16):
    w, b = dw.base, dw.base.batch
    bb = clone_batch(b, positions=None, adapter_ids=np.asarray(adapter_ids, np.int32))
    print(f"  [{what}] layers={w.model.n_layers} T={b.n_tokens} adapters={list(adapter_ids)}", flush=True)
    ctx = make_ctx(dw, adapters, max_rank)
    ctx.embed_txt(dw.token_ids, b.positions, b.in_embed_ids)
    pb = ctx.batch_create(bb)
    ctx.forward_all(pb)
    ctx.synchronize()
    stored = np.nonzero(b.out_embed_ids >= 0)[0]
    y_bits = ctx.embed_read(b.out_embed_ids[stored])
    kvs, emb = deep_oracle_pools(dw)
    O.embed_txt(dw.table_bits, dw.token_ids, b.positions, emb, b.in_embed_ids)
    res = O.forward_model(w.model, dw.layers, kvs, emb, b, round_intermediates=True, adapters=adapters,
                          adapter_ids=adapter_ids)
    assert_close(dec(y_bits), res[-1].y[stored], f"{what} output Embeds")
    pages, slots = appended_positions(w)
    k, v = ctx.kv_read(0, pages, slots)
    assert_bf16_close(k, res[0].k_new, f"{what} layer 0 appended K", ulps=2)
    assert_bf16_close(v, res[0].v_new, f"{what} layer 0 appended V", ulps=2)
    return ctx, y_bits, res, stored


def test_adapters_on_every_projection_mixed_batch():
    dw = W.deep_tiny(n_layers=2)
    m = dw.base.model
    adapters = {0: W.make_adapter(m, 6000, 0, rank=4, projections=ALL, scale=2.0, std=0.05),
                2: W.make_adapter(m, 6000, 2, rank=16, projections=("wq", "wv", "wup", "wdown"), scale=0.5, std=0.05)}
    ids = [0, -1, 2, 0, 2]  # four decode requests and the 32-token prefill
    ctx, y_ad, res, stored = compare(dw, adapters, ids, "tiny, two adapters")
    # the request without adapter gives the bits of a run without any adapter; the others differ
    b = dw.base.batch
    ctx0 = make_ctx(dw, {}, 0)
    ctx0.embed_txt(dw.token_ids, b.positions, b.in_embed_ids)
    pb0 = ctx0.batch_create(clone_batch(b, positions=None))
    ctx0.forward_all(pb0)
    ctx0.synchronize()
    y_plain = ctx0.embed_read(b.out_embed_ids[stored])
    req_of = np.searchsorted(b.tok_indptr, stored, side="right") - 1
    assert np.array_equal(y_ad[req_of == 1], y_plain[req_of == 1])
    assert not np.array_equal(y_ad[req_of == 0], y_plain[req_of == 0])
    assert not np.array_equal(y_ad[req_of == 4], y_plain[req_of == 4])


def test_adapter_head_dim_128_ragged():
    m = W.ModelDesc(hidden=256, n_q_heads=8, n_kv_heads=2, head_dim=128, mlp_dim=384, vocab=512, page_size=16,
                    rms_eps=1e-5, rope_theta=1e4, n_layers=3)
    reqs = [W.RequestSpec(1, 0), W.RequestSpec(2, 100), W.RequestSpec(33, 47), W.RequestSpec(1, 257, in_place=True)]
    dw = W.build_deep_workload("ad_ragged", m, reqs, n_kv_pages=64, seed=6500, std=0.05, resid_std=0.05 / np.sqrt(6.0))
    adapters = {1: W.make_adapter(m, 6500, 1, rank=7, projections=ALL, scale=1.0, std=0.05),
                3: W.make_adapter(m, 6500, 3, rank=3, projections=("wk", "wo", "wgate"), scale=4.0, std=0.05)}
    compare(dw, adapters, [1, 3, 1, -1], "D128 ragged, odd ranks", max_rank=8)


def test_adapter_many_rows_and_rank_blocks():
    """Adapter groups longer than one 32-row tile (prefill requests of 70 and 45 tokens, one adapter shared by a
    prefill and several decode requests), a rank above 32 (two blocks of rank columns) and one that is no
    multiple of 16, on every projection."""
    m = W.ModelDesc(hidden=256, n_q_heads=8, n_kv_heads=2, head_dim=64, mlp_dim=512, vocab=512, page_size=16,
                    rms_eps=1e-5, rope_theta=1e4, n_layers=2)
    reqs = [W.RequestSpec(70, 19), W.RequestSpec(1, 90, in_place=True), W.RequestSpec(45, 0), W.RequestSpec(1, 33),
            W.RequestSpec(2, 64), W.RequestSpec(1, 17), W.RequestSpec(33, 5)]
    dw = W.build_deep_workload("ad_rows", m, reqs, n_kv_pages=96, seed=6700, std=0.05, resid_std=0.05 / np.sqrt(4.0))
    adapters = {0: W.make_adapter(m, 6700, 0, rank=40, projections=ALL, scale=0.5, std=0.05),
                1: W.make_adapter(m, 6700, 1, rank=21, projections=ALL, scale=1.0, std=0.05)}
    compare(dw, adapters, [0, 0, 1, 1, 0, -1, -1], "tiles and rank blocks", max_rank=40)


def test_adapter_8b_shape_decode():
    """Rank-16 adapters on q, k, v, o (the usual targets) at the 8B widths, 16 decode requests, one layer."""
    m = W.model_8b()
    m.n_layers = 1
    ctxs = W.rng_for(6600, W.STREAM_CTX).integers(256, 1025, size=16)
    reqs = [W.RequestSpec(1, int(c), in_place=True) for c in ctxs]
    dw = W.build_deep_workload("ad_8b", m, reqs, n_kv_pages=1200, seed=6600, std=0.02, resid_std=0.02 / 8.0)
    adapters = {0: W.make_adapter(m, 6600, 0, rank=16, projections=("wq", "wk", "wv", "wo"), scale=2.0),
                1: W.make_adapter(m, 6600, 1, rank=16, projections=("wq", "wk", "wv", "wo"), scale=2.0)}
    ids = [i % 3 - 1 for i in range(16)]  # -1, 0, 1, ...
    compare(dw, adapters, ids, "8B shape, rank 16 on q/k/v/o")


def test_adapter_error_codes():
    from paper_2510_24051_amd import Pie, PieError
    dw = W.deep_tiny(n_layers=1)
    m, b = dw.base.model, dw.base.batch
    ad = W.make_adapter(m, 1, 0, rank=4, projections=("wq",))

    def status_of(fn):
        with pytest.raises(PieError) as e:
            fn()
        return e.value.status
    plain = make_ctx(dw, {}, 0)
    assert status_of(lambda: plain.load_adapter(0, ad)) == -1                     # context without adapters
    plain.embed_txt(dw.token_ids, b.positions, b.in_embed_ids)
    assert status_of(lambda: plain.batch_create(clone_batch(b, adapter_ids=np.zeros(b.n_requests, np.int32)))) == -2
    plain.batch_create(clone_batch(b, adapter_ids=np.full(b.n_requests, -1, np.int32))).destroy()  # "none" is fine
    ctx = make_ctx(dw, {0: ad}, 4)
    assert status_of(lambda: ctx.load_adapter(1, ad)) == -2                       # adapter index out of range
    big = W.make_adapter(m, 1, 0, rank=5, projections=("wq",))
    assert status_of(lambda: ctx.load_adapter(0, big)) == -2                      # rank above max_lora_rank
    assert status_of(lambda: ctx.load_adapter(0, [ad[0], ad[0]])) == -2           # layer out of range
    ctx.embed_txt(dw.token_ids, b.positions, b.in_embed_ids)
    assert status_of(lambda: ctx.batch_create(clone_batch(b, adapter_ids=np.full(b.n_requests, 1, np.int32)))) == -2
    assert status_of(lambda: ctx.batch_create(clone_batch(b, adapter_ids=np.full(b.n_requests, -2, np.int32)))) == -2
