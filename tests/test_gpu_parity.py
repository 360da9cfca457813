"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Tolerances: layer outputs (bf16) max-abs <= 2e-2 and mean-abs <= 2e-3 against the oracle's wide value;
integer/byte work (pool round trips, page slots, top-k ids outside logit ties < 1e-3) exact."""
import copy

import numpy as np
import pytest

import workloads as W
from oracle import pie_oracle as O
from gpu_helpers import (appended_positions, assert_bf16_close, assert_close, assert_y_close, dec, gpu_forward, make_ctx,
                         seed_ctx)
from helpers import check_topk, oracle_pools, run_oracle

pytestmark = pytest.mark.gpu


def small_model(head_dim=64, n_q=4, n_kv=2, hidden=128, mlp=256, vocab=512):
    return W.ModelDesc(hidden=hidden, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=head_dim, mlp_dim=mlp, vocab=vocab,
                       page_size=16, rms_eps=1e-5, rope_theta=1e4, n_layers=1)


def random_mask(p):
    def f(n_new, L, rng):
        m = rng.random((n_new, L)) < p
        m &= W.causal_bitmap(n_new, L)
        return m
    return f


def compare_layer(w, ctx=None, mode_b_only=False, check_taps=True, what=""):
    """Full element-by-element comparison of one forward call (outputs, taps, appended KV)."""
    ctx = ctx or make_ctx(w)
    pb, stored, y_bits = gpu_forward(ctx, w)
    T = w.batch.n_tokens
    res_b, kv_b, _ = run_oracle(w, round_intermediates=True)
    assert_y_close(dec(y_bits), res_b.y[stored], f"{what} y vs oracle (bf16 intermediates)")
    if not mode_b_only:
        res_a, _, _ = run_oracle(w)
        assert_y_close(dec(y_bits), res_a.y[stored], f"{what} y vs oracle (wide intermediates)", stored_as=res_b.y[stored])
    if check_taps:
        from paper_2510_24051_amd import TAP_ACT, TAP_ATTN, TAP_Q, TAP_RESID
        m = w.model
        q = dec(ctx.read_tap(TAP_Q, T)).reshape(T, m.n_q_heads, m.head_dim)
        assert_close(q, res_b.q, f"{what} q after rotary step", 4e-2 * max(1.0, np.abs(res_b.q).max() / 4), 2e-3 * max(1.0, np.abs(res_b.q).mean()))
        o = dec(ctx.read_tap(TAP_ATTN, T)).reshape(T, m.n_q_heads, m.head_dim)
        assert_close(o, res_b.o, f"{what} attention output", 2e-2 * max(1.0, np.abs(res_b.o).max()), 2e-3 * max(1.0, np.abs(res_b.o).mean() * 4))
        h = ctx.read_tap(TAP_RESID, T)
        assert_close(h, res_b.h, f"{what} residual after attention")
        act = dec(ctx.read_tap(TAP_ACT, T))
        assert_close(act, res_b.act, f"{what} SwiGLU activation", 2e-2 * max(1.0, np.abs(res_b.act).max()),
                     2e-3 * max(1.0, np.abs(res_b.act).mean() * 4))
    # appended K/V land in the right (page, slot), values equal up to bf16 rounding of an fp32 vs fp64 product
    pages, slots = appended_positions(w)
    k_gpu, v_gpu = ctx.kv_read(0, pages, slots)
    assert_bf16_close(k_gpu, res_b.k_new, f"{what} appended K", ulps=2)
    assert_bf16_close(v_gpu, res_b.v_new, f"{what} appended V", ulps=2)
    # prior KV untouched (byte work: exact)
    if len(w.prior.page_ids):
        k0, v0 = ctx.kv_read(0, w.prior.page_ids, w.prior.slots)
        assert np.array_equal(k0, w.prior.k_bits) and np.array_equal(v0, w.prior.v_bits)
    return ctx, pb, y_bits, stored


def compare_dist(ctx, w, what=""):
    """get_next_dist on the GPU's own stored output Embeds (the resource boundary between the two calls)."""
    ids_e = w.batch.out_embed_ids[w.dist_rows]
    gi, gp = ctx.get_next_dist(ids_e, w.top_k, w.temperature)
    emb = O.EmbedPool(w.n_embeds, w.model.hidden)
    emb.write(ids_e, ctx.embed_read(ids_e))
    oi, op, z = O.get_next_dist(w.model, w.head, emb, ids_e, w.top_k, w.temperature, round_intermediates=True)
    check_topk(gi, gp, z / w.temperature, oi, op)
    from paper_2510_24051_amd import TAP_LOGITS
    zg = ctx.read_tap(TAP_LOGITS, len(ids_e))
    mx = np.abs(zg - z).max()
    print(f"    {what} logits max-abs {mx:.3e}; ids equal {np.mean(gi == oi) * 100:.2f}%", flush=True)
    assert mx < 1e-3


# ---------------------------------------------------------------- byte work
def test_pool_roundtrips_are_bit_exact():
    m = small_model()
    w = W.build_workload("rt", m, [W.RequestSpec(3, 40), W.RequestSpec(1, 7)], n_kv_pages=16, seed=1)
    ctx = make_ctx(w)
    assert np.array_equal(ctx.embed_read(w.batch.in_embed_ids), w.embed_bits)
    k, v = ctx.kv_read(0, w.prior.page_ids, w.prior.slots)
    assert np.array_equal(k, w.prior.k_bits) and np.array_equal(v, w.prior.v_bits)
    untouched = np.setdiff1d(np.arange(w.n_embeds), w.batch.in_embed_ids)
    assert not ctx.embed_read(untouched).any()


# ---------------------------------------------------------------- config 1
def test_c1_tiny_layer_and_dist():
    w = W.c1_tiny()
    ctx, pb, y_bits, stored = compare_layer(w, what="c1")
    compare_dist(ctx, w, "c1")
    # explicit causal bitmaps give the same bits as inferred causal masks
    wb = W.c1_tiny(bitmap=True)
    ctx2 = make_ctx(wb)
    _, _, y2 = gpu_forward(ctx2, wb)
    assert np.array_equal(y2, y_bits)


def test_c1_literal_unstored_rows_and_in_place():
    w = W.c1_tiny()
    w2 = copy.deepcopy(w)
    b = w2.batch
    t0 = b.tok_indptr[4]
    b.out_embed_ids[t0:t0 + 31] = -1  # prefill keeps only its last row
    ctx = make_ctx(w2)
    before = ctx.embed_read(np.arange(w2.n_embeds))
    _, stored, y_bits = gpu_forward(ctx, w2)
    res, _, _ = run_oracle(w2, round_intermediates=True)
    assert_close(dec(y_bits), res.y[stored], "c1 stored rows")
    after = ctx.embed_read(np.arange(w2.n_embeds))
    changed = np.nonzero((before != after).any(axis=1))[0]
    assert set(changed.tolist()) <= set(b.out_embed_ids[stored].tolist())


# ---------------------------------------------------------------- ragged shapes, masks, head dims, group sizes
@pytest.mark.parametrize("head_dim,n_q,n_kv", [(64, 4, 2), (128, 8, 2), (128, 8, 1), (64, 2, 2), (64, 8, 1)])
def test_ragged_mixed_batch(head_dim, n_q, n_kv):
    m = small_model(head_dim, n_q, n_kv)
    sparse = random_mask(0.3)
    reqs = [W.RequestSpec(1, 0), W.RequestSpec(1, 15), W.RequestSpec(1, 16), W.RequestSpec(2, 100),
            W.RequestSpec(3, 33, mask=sparse), W.RequestSpec(9, 0), W.RequestSpec(31, 5, mask=W.causal_bitmap),
            W.RequestSpec(33, 47), W.RequestSpec(70, 130, mask=sparse), W.RequestSpec(1, 700, mask=random_mask(0.02)),
            W.RequestSpec(1, 257, in_place=True), W.RequestSpec(40, 0, mask=random_mask(0.9))]
    w = W.build_workload("ragged", m, reqs, n_kv_pages=160, seed=100 + head_dim + n_q, std=0.05)
    compare_layer(w, what=f"ragged D{head_dim} {n_q}/{n_kv}")


@pytest.mark.parametrize("hidden,mlp,n_q,n_kv,T_prefill", [(256, 320, 6, 2, 290), (192, 512, 4, 2, 600),
                                                          (256, 512, 4, 4, 513), (256, 256, 8, 2, 1100)])
def test_large_batches_on_small_models(hidden, mlp, n_q, n_kv, T_prefill):
    """More than 256 rows: the tiled GEMM kernels (both the asynchronous-copy one and the one for contraction
    lengths that are not a multiple of 128) on ragged row counts and output widths that do not fill a tile."""
    m = small_model(64, n_q, n_kv, hidden=hidden, mlp=mlp, vocab=512)
    reqs = [W.RequestSpec(T_prefill, 21), W.RequestSpec(1, 50), W.RequestSpec(1, 0), W.RequestSpec(3, 10)]
    w = W.build_workload("large", m, reqs, n_kv_pages=128, seed=300 + hidden + mlp, std=0.05)
    compare_layer(w, what=f"T={w.batch.n_tokens} H{hidden} I{mlp} {n_q}/{n_kv}")


@pytest.mark.parametrize("n_decode,n_prefill", [(40, 60), (100, 0), (57, 143), (129, 0), (64, 192), (1, 64)])
def test_mid_size_batches_split_k_tiles(n_decode, n_prefill):
    """65 to 256 rows on a model whose contraction lengths (1024, 2048) are long enough for the tiled GEMM to split
    them across workgroups: 128-row tiles up to 128 rows, 256-row tiles above, ragged row counts in both, the
    partial sums taken by the split-K epilogue, the rotary step and the second norm."""
    m = small_model(64, 16, 4, hidden=1024, mlp=2048, vocab=512)
    rng = np.random.default_rng(n_decode * 1000 + n_prefill)
    reqs = [W.RequestSpec(1, int(c)) for c in rng.integers(0, 60, size=n_decode)]
    if n_prefill:
        reqs.append(W.RequestSpec(n_prefill, 7))
    w = W.build_workload("mid", m, reqs, n_kv_pages=n_decode * 4 + 32, seed=900 + n_decode + n_prefill, std=0.012)
    compare_layer(w, what=f"T={w.batch.n_tokens} H1024 I2048")


@pytest.mark.parametrize("mlp,n_decode", [(24576, 12), (24608, 40), (24576, 64), (12320, 40), (12288, 12)])
def test_wide_mlp_gate_up_without_split(mlp, n_decode):
    """An MLP wide enough that the gate/up product fills the chip with one 32-column block per wave and no split
    along K: the gate block of a pair and its up block sit in neighbouring waves and meet through LDS.  24608 is
    32 x 769: the last workgroup has two idle waves that still have to take part in the exchange's barrier.  Half
    that width runs the same scheme with workgroups of two waves (one pair each)."""
    m = small_model(64, 4, 2, hidden=128, mlp=mlp, vocab=512)
    rng = np.random.default_rng(mlp + n_decode)
    reqs = [W.RequestSpec(1, int(c)) for c in rng.integers(0, 40, size=n_decode)]
    w = W.build_workload("wide_mlp", m, reqs, n_kv_pages=n_decode * 3 + 8, seed=950 + n_decode, std=0.02,
                         resid_std=0.02 / np.sqrt(mlp / 128.0))
    compare_layer(w, what=f"T={w.batch.n_tokens} I{mlp}")


# ---------------------------------------------------------------- shared prefixes (requests aliasing pages)
def hide_span(a0, a1):
    def f(n_new, L, rng):
        m = W.causal_bitmap(n_new, L)
        m[:, a0:a1] = False
        return m
    return f


@pytest.mark.parametrize("head_dim,n_q,n_kv", [(64, 4, 2), (128, 8, 2), (64, 2, 2)])
def test_shared_prefix_requests_are_grouped_and_match(head_dim, n_q, n_kv):
    """Requests whose page tables alias the same prefix pages: the decode kernel reads each shared K/V block
    once for several requests (fewer bytes requested than the per-request count), same result as the oracle,
    which gathers every request's KV separately."""
    m = small_model(head_dim, n_q, n_kv)
    P = 16
    reqs = [W.RequestSpec(1, 5 * P + 3, prefix_group=0, prefix_len=5 * P),                       # causal
            W.RequestSpec(1, 5 * P + 40, prefix_group=0, prefix_len=5 * P, mask=hide_span(P, 3 * P)),  # hides pages 1-2
            W.RequestSpec(1, 5 * P, prefix_group=0, prefix_len=5 * P, in_place=True),            # no private prior
            W.RequestSpec(1, 9 * P + 1, prefix_group=0, prefix_len=5 * P, mask=W.causal_bitmap),
            W.RequestSpec(1, 5 * P + 7, prefix_group=0, prefix_len=5 * P, mask=random_mask(0.2)),
            W.RequestSpec(1, 33),                                                              # unrelated
            W.RequestSpec(2, 3 * P + 5, prefix_group=1, prefix_len=3 * P),                       # two rows per head
            W.RequestSpec(2, 3 * P + 20, prefix_group=1, prefix_len=3 * P, mask=hide_span(0, 20)),
            W.RequestSpec(1, 6 * P, prefix_group=0, prefix_len=5 * P),
            W.RequestSpec(40, 3 * P, prefix_group=1, prefix_len=3 * P),                          # prefill over a shared prefix
            W.RequestSpec(1, 2 * P + 2, prefix_group=2, prefix_len=2 * P),
            W.RequestSpec(1, 2 * P + 9, prefix_group=2, prefix_len=2 * P)]
    w = W.build_workload("shared", m, reqs, n_kv_pages=96, seed=700 + head_dim + n_q, std=0.05)
    ctx, pb, _, _ = compare_layer(w, what=f"shared prefixes D{head_dim} {n_q}/{n_kv}")
    work = pb.work()
    print(f"    decode KV bytes: per request {work['kv_bytes_decode']}, requested {work['kv_bytes_requested']}, "
          f"distinct pages {work['kv_bytes_unique']}", flush=True)
    assert work["kv_bytes_requested"] < work["kv_bytes_decode"]


def test_partially_shared_tables_and_tables_in_another_order():
    """Same first page, one differing page in the middle (only the equal positions are shared); and two
    requests naming the same prefix pages in a different logical order (only position 0 matches: nothing is
    grouped, the result is still the oracle's)."""
    m = small_model()
    P = 16
    reqs = [W.RequestSpec(1, 4 * P + 5, prefix_group=0, prefix_len=4 * P),
            W.RequestSpec(1, 4 * P + 9, prefix_group=0, prefix_len=4 * P),
            W.RequestSpec(1, 4 * P + 1, prefix_group=0, prefix_len=4 * P),
            W.RequestSpec(1, 3 * P + 4, prefix_group=1, prefix_len=3 * P),
            W.RequestSpec(1, 3 * P + 11, prefix_group=1, prefix_len=3 * P)]
    w = W.build_workload("partial", m, reqs, n_kv_pages=64, seed=77, std=0.05)
    b = w.batch
    used = set(b.page_ids.tolist())
    spare = [p for p in range(64) if p not in used]
    # request 1: logical page 2 becomes a private page with contents of its own
    rng = W.rng_for(77, 99)
    b.page_ids[b.page_indptr[1] + 2] = spare[0]
    w.prior.page_ids = np.concatenate([w.prior.page_ids, np.full(P, spare[0], np.int32)])
    w.prior.slots = np.concatenate([w.prior.slots, np.arange(P, dtype=np.int32)])
    w.prior.k_bits = np.concatenate([w.prior.k_bits, W.normal_bf16(rng, (P, m.n_kv_heads, m.head_dim))])
    w.prior.v_bits = np.concatenate([w.prior.v_bits, W.normal_bf16(rng, (P, m.n_kv_heads, m.head_dim))])
    # request 4 reads the shared prefix pages 1 and 2 in the other order
    a4 = b.page_indptr[4]
    b.page_ids[a4 + 1], b.page_ids[a4 + 2] = b.page_ids[a4 + 2], b.page_ids[a4 + 1]
    ctx, pb, _, _ = compare_layer(w, what="partially shared tables")
    work = pb.work()
    # requests 0-2 share logical pages 0, 1, 3 (3 pages read once instead of three times); 3-4 share nothing
    page_bytes = m.n_kv_heads * 2 * P * m.head_dim * 2
    assert work["kv_bytes_decode"] - work["kv_bytes_requested"] == 2 * 3 * page_bytes


def test_rows_without_visible_keys_output_the_residual_only():
    m = small_model()

    def none_visible(n_new, L, rng):
        a = W.causal_bitmap(n_new, L)
        a[0, :] = False
        return a
    reqs = [W.RequestSpec(1, 20, mask=none_visible), W.RequestSpec(40, 3, mask=none_visible)]
    w = W.build_workload("blind", m, reqs, n_kv_pages=16, seed=5, std=0.05)
    ctx, *_ = compare_layer(w, what="blind rows")
    from paper_2510_24051_amd import TAP_ATTN
    o = ctx.read_tap(TAP_ATTN, w.batch.n_tokens)
    assert not o[0].any() and not o[1].any()


def test_sparse_mask_skips_pages_and_matches():
    m = small_model(128, 8, 2)
    reqs = [W.RequestSpec(1, 1500, mask=W.sink_window_mask(4, 100)), W.RequestSpec(2, 900, mask=W.sink_window_mask(4, 64))]
    w = W.build_workload("sinkwin", m, reqs, n_kv_pages=200, seed=6, std=0.05)
    ctx, pb, *_ = compare_layer(w, what="sink+window")
    work = pb.work()
    assert work["visited_pages"] == (1 + 7) + (1 + 5)  # sink page + window pages only
    assert work["kv_bytes"] == work["visited_pages"] * 2 * 16 * 128 * 2 * 2


def test_split_call_equivalence_on_gpu():
    m = small_model()
    one = W.build_workload("split", m, [W.RequestSpec(40, 0)], n_kv_pages=8, seed=21, std=0.05)
    ctx = make_ctx(one)
    _, _, y_one = gpu_forward(ctx, one)
    b = one.batch
    ctx2 = make_ctx(one)
    from helpers import clone_batch
    first = clone_batch(b, n_tokens=39, tok_indptr=np.array([0, 39], np.int32), in_embed_ids=b.in_embed_ids[:39],
                        out_embed_ids=np.full(39, -1, np.int32), positions=b.positions[:39],
                        kv_len=np.array([39], np.int32))
    ctx2.forward_host(0, first)
    second = clone_batch(b, n_tokens=1, tok_indptr=np.array([0, 1], np.int32), in_embed_ids=b.in_embed_ids[39:],
                         out_embed_ids=b.out_embed_ids[39:], positions=b.positions[39:],
                         kv_len=np.array([40], np.int32))
    ctx2.forward_host(0, second)
    y_two = ctx2.embed_read(b.out_embed_ids[39:])
    assert_close(dec(y_two), dec(y_one[39:]), "split call vs single call", 2e-2, 2e-3)
    pages, slots = appended_positions(one)
    k1, v1 = ctx.kv_read(0, pages, slots)
    k2, v2 = ctx2.kv_read(0, pages, slots)
    assert np.array_equal(k1, k2) and np.array_equal(v1, v2)


def test_batch_composition_invariance_on_gpu():
    m = small_model()
    reqs = [W.RequestSpec(1, 90), W.RequestSpec(35, 10), W.RequestSpec(2, 300)]
    w = W.build_workload("comp", m, reqs, n_kv_pages=64, seed=33, std=0.05)
    ctx = make_ctx(w)
    _, _, y_all = gpu_forward(ctx, w)
    b = w.batch
    from helpers import clone_batch
    for r in range(3):
        a, e = b.tok_indptr[r], b.tok_indptr[r + 1]
        pa, pe = b.page_indptr[r], b.page_indptr[r + 1]
        solo = clone_batch(b, n_requests=1, n_tokens=e - a, tok_indptr=np.array([0, e - a], np.int32),
                           in_embed_ids=b.in_embed_ids[a:e], out_embed_ids=b.out_embed_ids[a:e],
                           positions=b.positions[a:e], page_indptr=np.array([0, pe - pa], np.int32),
                           page_ids=b.page_ids[pa:pe], kv_len=b.kv_len[r:r + 1])
        c2 = make_ctx(w)
        c2.forward_host(0, solo)
        y = c2.embed_read(b.out_embed_ids[a:e])
        # GEMM tiling depends on the row count, so allow rounding-level differences only
        assert_close(dec(y), dec(y_all[a:e]), f"request {r} alone vs in batch", 2e-2, 5e-4)


# ---------------------------------------------------------------- distribution
@pytest.mark.parametrize("k,temp", [(1, 1.0), (8, 0.7), (256, 1.0), (300, 2.0)])
def test_get_next_dist_top_k(k, temp):
    m = small_model(vocab=2048)
    w = W.build_workload("dist", m, [W.RequestSpec(1, 5) for _ in range(7)], n_kv_pages=16, seed=40, std=0.05,
                         top_k=k, temperature=temp)
    ctx = make_ctx(w, max_top_k=512)
    gpu_forward(ctx, w)
    compare_dist(ctx, w, f"k={k} T={temp}")


@pytest.mark.parametrize("vocab,k", [(131072, 1024), (131072, 1), (32, 32), (8192, 1000), (8224, 7)])
def test_get_next_dist_size_limits(vocab, k):
    """Largest vocabulary and K the kernels take, K equal to the vocabulary, a vocabulary of exactly one chunk and
    one that spills 32 entries into a second chunk."""
    m = small_model(vocab=vocab)
    w = W.build_workload("dist_lim", m, [W.RequestSpec(1, 5) for _ in range(3)], n_kv_pages=8, seed=42, std=0.05,
                         top_k=k)
    ctx = make_ctx(w, max_top_k=1024)
    gpu_forward(ctx, w)
    compare_dist(ctx, w, f"V={vocab} k={k}")
    if k == vocab:
        _, gp = ctx.get_next_dist(w.batch.out_embed_ids[w.dist_rows], k, 1.0)
        np.testing.assert_allclose(gp.sum(axis=1), 1.0, rtol=1e-5)


def test_get_next_dist_many_rows_long_chunks():
    """Enough rows that the chunk kernel takes 16384-logit chunks (two of them for 16416 logits, the second with
    32 entries), K larger than the short chunk."""
    m = small_model(vocab=16416)
    w = W.build_workload("dist_rows", m, [W.RequestSpec(1, 3) for _ in range(360)], n_kv_pages=400, seed=43, std=0.05,
                         top_k=40)
    ctx = make_ctx(w, max_top_k=64)
    gpu_forward(ctx, w)
    compare_dist(ctx, w, "360 rows, V=16416, k=40")


def test_top_k_ties_pick_lower_ids():
    m = small_model(vocab=512)
    w = W.build_workload("ties", m, [W.RequestSpec(1, 3)], n_kv_pages=4, seed=41, std=0.05, top_k=40)
    w.head.w_lm[:] = 0  # all logits equal -> ids 0..k-1, uniform probabilities
    ctx = make_ctx(w)
    gpu_forward(ctx, w)
    gi, gp = ctx.get_next_dist(w.batch.out_embed_ids[:1], 40, 1.0)
    assert gi[0].tolist() == list(range(40))
    np.testing.assert_allclose(gp[0], 1.0 / 512, rtol=1e-5)


@pytest.mark.parametrize("vocab,k", [(16384, 40), (65536, 300)])
def test_top_k_ties_in_long_rows(vocab, k):
    """All logits equal in rows of several chunks: every key shares the top byte of the k-th largest, so the chunk
    kernel's short list overflows and the selection over all keys in registers runs, with the cut inside the tie."""
    m = small_model(vocab=vocab)
    w = W.build_workload("ties_long", m, [W.RequestSpec(1, 3), W.RequestSpec(1, 2)], n_kv_pages=4, seed=44, std=0.05,
                         top_k=k)
    w.head.w_lm[:] = 0
    ctx = make_ctx(w, max_top_k=512)
    gpu_forward(ctx, w)
    gi, gp = ctx.get_next_dist(w.batch.out_embed_ids[:2], k, 1.0)
    for r in range(2):
        assert gi[r].tolist() == list(range(k))
    np.testing.assert_allclose(gp, 1.0 / vocab, rtol=1e-5)


def crafted_logit_rows(vocab, rows):
    """A context whose get_next_dist returns exactly the given logit rows (bf16 values): no final norm, Embed r is
    the r-th unit vector and column r of the LM head holds row r."""
    H = 128
    m = small_model(hidden=H, vocab=vocab)
    w = W.build_workload("crafted", m, [W.RequestSpec(1, 3) for _ in range(len(rows))], n_kv_pages=16, seed=45,
                         std=0.05, top_k=256)
    w.head.g_final = None
    w.head.w_lm[:] = 0
    for r, z in enumerate(rows):
        w.head.w_lm[:, r] = W.to_bf16_bits(np.asarray(z, dtype=np.float32))
    ctx = make_ctx(w, max_top_k=256, max_dist_rows=len(rows))
    unit = np.zeros((len(rows), H), dtype=np.float32)
    unit[np.arange(len(rows)), np.arange(len(rows))] = 1.0
    ids = np.arange(len(rows), dtype=np.int32)
    ctx.embed_write(ids, W.to_bf16_bits(unit))
    return ctx, w, ids


def test_top_k_across_the_sign_boundary_is_exact_and_no_slower():
    """Rows whose maximum is positive and whose k-th largest is negative (the order keys of the two lie 128 top-byte
    values apart), and rows shifted to mean -8 with a handful of positive logits: same exact result as the oracle's
    full sort, and the top-k kernels take about as long as on a N(0,1) row."""
    V, k = 128256, 256
    rng = np.random.default_rng(46)
    plain = rng.standard_normal(V)
    shifted = rng.standard_normal(V) - 8.0
    shifted[rng.choice(V, 5, replace=False)] = rng.random(5) * 3 + 0.5       # k-th largest is about -5
    mixed = rng.standard_normal(V) * 0.5 - 3.0
    mixed[rng.choice(V, 100, replace=False)] = rng.random(100) * 2 + 1.0     # 100 positives, the rest negative
    tiny = np.where(rng.random(V) < 0.5, 1.0, -1.0) * 10.0 ** rng.uniform(-30, 0, V)  # every exponent in use
    rows = [plain, shifted, mixed, tiny]
    ctx, w, ids = crafted_logit_rows(V, rows)
    gi, gp = ctx.get_next_dist(ids, k, 1.0)
    z = np.stack([dec(W.to_bf16_bits(np.asarray(r, dtype=np.float32))) for r in rows])
    oi, op = O.top_k_dist(z, k, 1.0)
    assert np.array_equal(gi, oi)  # crafted logits are exact on both sides: no tie slack needed
    np.testing.assert_allclose(gp, op, rtol=2e-3, atol=1e-12)
    # one row at a time, stage-timed: the walk from the maximum's top byte must not take longer across the boundary
    ctx.set_stage_timing(True)
    t = []
    for r in range(len(rows)):
        samples = []
        for _ in range(7):
            ctx.get_next_dist(ids[r:r + 1], k, 1.0)
            samples.append(ctx.stage_times()["topk"])
        t.append(float(np.median(samples)))
    ctx.set_stage_timing(False)
    print(f"    top-k of one row of {V}: N(0,1) {t[0] * 1e3:.1f} us, mean -8 with 5 positives {t[1] * 1e3:.1f} us, "
          f"100 positives over negatives {t[2] * 1e3:.1f} us, all exponents {t[3] * 1e3:.1f} us", flush=True)
    assert max(t[1:]) <= 2.0 * t[0]
    ctx.close()


# ---------------------------------------------------------------- error paths (detected on the host)
def test_error_codes():
    from paper_2510_24051_amd import Pie, PieError
    m = small_model()
    w = W.build_workload("err", m, [W.RequestSpec(2, 10), W.RequestSpec(1, 4)], n_kv_pages=8, seed=50, std=0.05, top_k=4)
    ctx = make_ctx(w)

    def status_of(fn):
        with pytest.raises(PieError) as e:
            fn()
        return e.value.status
    b = copy.deepcopy(w.batch)
    b.page_ids[0] = 99
    assert status_of(lambda: ctx.batch_create(b)) == -2  # PIE_ERANGE
    b = copy.deepcopy(w.batch)
    b.in_embed_ids[0] = w.n_embeds
    assert status_of(lambda: ctx.batch_create(b)) == -2
    b = copy.deepcopy(w.batch)  # second request writes the slot of the first one's last token
    b.page_ids[b.page_indptr[1]] = b.page_ids[0]
    b.kv_len[1] = 12
    assert status_of(lambda: ctx.batch_create(b, validate=True)) == -4  # PIE_ECONFLICT
    big = W.build_workload("big", m, [W.RequestSpec(4, 0)], n_kv_pages=8, seed=51, std=0.05)
    assert status_of(lambda: ctx.batch_create(big.batch)) == -3  # PIE_EBATCH: 4 tokens > 3
    assert status_of(lambda: ctx.get_next_dist([0], 0)) == -2
    assert status_of(lambda: ctx.get_next_dist([0], 4, temperature=0.0)) == -1
    assert status_of(lambda: ctx.get_next_dist([w.n_embeds], 4)) == -2
    assert status_of(lambda: ctx.embed_read([-1])) == -2
    assert status_of(lambda: ctx.kv_read(0, [0], [16])) == -2
    bad = copy.copy(m)
    bad.page_size = 8
    with pytest.raises(PieError) as e:
        Pie(bad, 8, 8, 4, 4)
    assert e.value.status == -7  # PIE_EUNSUPPORTED
    # a batch of another context, or of a planning context (no device block), is refused before anything is launched
    other = make_ctx(w)
    pb_other = other.batch_create(w.batch)
    assert ctx.lib.pie_forward(ctx.ctx, 0, pb_other.handle) == -1 and ctx.lib.pie_forward_all(ctx.ctx, pb_other.handle) == -1
    assert ctx.lib.pie_batch_destroy(ctx.ctx, pb_other.handle) == -1
    pb_other.destroy()
    other.close()
    planner = Pie.planner(m, w.n_kv_pages, w.n_embeds, 3, 2)
    pb_plan = planner.batch_create(w.batch)
    assert ctx.lib.pie_forward(ctx.ctx, 0, pb_plan.handle) == -1
    pb_plan.destroy()
    planner.close()
    # the context still works after the failed calls
    compare_layer(w, ctx=ctx, what="after errors")
