"""The allocation-free entry point pie_get_next_dist_static against pie_get_next_dist: same kernels on a static
device array instead of the context's workspace, so ids and probabilities must be identical; and both against the
oracle.  Two calls in a row on one GPU, the second with a smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import pie_oracle as O
from gpu_helpers import gpu_forward, make_ctx
from helpers import check_topk

pytestmark = pytest.mark.gpu


def both(ctx, ids_e, k, temp):
    n = len(ids_e)
    oi = torch.full((n, k), -7, dtype=torch.int32, device=ctx.device)
    op = torch.full((n, k), -7.0, dtype=torch.float32, device=ctx.device)
    ctx.get_next_dist_static_async(ids_e, k, temp, oi, op)
    ctx.synchronize()
    si, sp = oi.cpu().numpy(), op.cpu().numpy()
    gi, gp = ctx.get_next_dist(ids_e, k, temp)
    return si, sp, gi, gp


def test_static_scratch_variant_equals_the_allocating_one():
    from paper_2510_24051_amd import PieError
    m = W.ModelDesc(hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, mlp_dim=512, vocab=40032, page_size=16,
                    rms_eps=1e-5, rope_theta=1e4, n_layers=1)
    w = W.build_workload("static", m, [W.RequestSpec(1, 5) for _ in range(32)], n_kv_pages=64, seed=61, std=0.05,
                         top_k=300)
    ctx = make_ctx(w, max_top_k=512, max_dist_rows=32)
    gpu_forward(ctx, w)
    ids_all = w.batch.out_embed_ids[w.dist_rows]
    for ids_e, k, temp in ((ids_all, 300, 1.0), (ids_all[3:8], 17, 0.6)):  # the second call is smaller
        si, sp, gi, gp = both(ctx, ids_e, k, temp)
        assert np.array_equal(si, gi) and np.array_equal(sp, gp)
        emb = O.EmbedPool(w.n_embeds, m.hidden)
        emb.write(ids_e, ctx.embed_read(ids_e))
        oi, op, z = O.get_next_dist(m, w.head, emb, ids_e, k, temp, round_intermediates=True)
        check_topk(si, sp, z / temp, oi, op)
    # limits are refused with an error, nothing is launched
    oi = torch.empty((33, 4), dtype=torch.int32, device=ctx.device)
    op = torch.empty((33, 4), dtype=torch.float32, device=ctx.device)
    with pytest.raises(PieError) as e:
        ctx.get_next_dist_static_async(np.arange(33, dtype=np.int32), 4, 1.0, oi, op)
    assert e.value.status == -3  # PIE_EBATCH: more than 32 rows
    with pytest.raises(PieError) as e:
        ctx.get_next_dist_static_async([w.n_embeds], 4, 1.0, oi, op)
    assert e.value.status == -2
    with pytest.raises(PieError) as e:
        ctx.get_next_dist_static_async([0], 0, 1.0, oi, op)
    assert e.value.status == -2
    ctx.close()


def test_static_scratch_size_limit_and_a_second_context():
    """The largest vocabulary: 32 rows of logits alone fill the 16 MiB array, so the call is refused; 24 rows with
    the largest top_k fit.  A second context on the same GPU uses the same array after the first."""
    from paper_2510_24051_amd import PieError
    m = W.ModelDesc(hidden=128, n_q_heads=2, n_kv_heads=2, head_dim=64, mlp_dim=256, vocab=131072, page_size=16,
                    rms_eps=1e-5, rope_theta=1e4, n_layers=1)
    w = W.build_workload("static_big", m, [W.RequestSpec(1, 3) for _ in range(32)], n_kv_pages=64, seed=62, std=0.05,
                         top_k=1024)
    ctx = make_ctx(w, max_top_k=1024, max_dist_rows=32)
    gpu_forward(ctx, w)
    ids_all = w.batch.out_embed_ids[w.dist_rows]
    oi = torch.empty((32, 1024), dtype=torch.int32, device=ctx.device)
    op = torch.empty((32, 1024), dtype=torch.float32, device=ctx.device)
    with pytest.raises(PieError) as e:  # 32 x 131072 x 4 B of logits = 16 MiB, plus candidates
        ctx.get_next_dist_static_async(ids_all, 1024, 1.0, oi, op)
    assert e.value.status == -3
    si, sp, gi, gp = both(ctx, ids_all[:24], 1024, 1.0)
    assert np.array_equal(si, gi) and np.array_equal(sp, gp)
    ctx2 = make_ctx(w, max_top_k=64, max_dist_rows=4)
    gpu_forward(ctx2, w)
    si, sp, gi, gp = both(ctx2, ids_all[:2], 5, 2.0)
    assert np.array_equal(si, gi) and np.array_equal(sp, gp)
    ctx.close()
    ctx2.close()
