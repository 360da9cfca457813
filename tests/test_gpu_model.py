"""GPU parity (through the C ABI) for `embed_txt` and for `forward` through every layer of a model:
the HIP path against the CPU oracle's `embed_txt` / `forward_model` on the same seeded inputs."""
import copy

import numpy as np
import pytest

import workloads as W
from oracle import pie_oracle as O
from helpers import check_topk, clone_batch, deep_oracle_pools
from gpu_helpers import appended_positions, assert_bf16_close, assert_close, dec

pytestmark = pytest.mark.gpu


def make_deep_ctx(dw, load_table=True, max_batch_tokens=None):
    from paper_2510_24051_amd import Pie
    w, b = dw.base, dw.base.batch
    ctx = Pie(w.model, w.n_kv_pages, w.n_embeds, max_batch_tokens=max_batch_tokens or b.n_tokens,
              max_batch_requests=b.n_requests, max_top_k=256, max_dist_rows=max(len(w.dist_rows), 1),
              n_layers=w.model.n_layers)
    for l, lw in enumerate(dw.layers):
        ctx.load_layer(l, lw)
    ctx.load_head(w.head)
    if load_table:
        ctx.load_embedding(dw.table_bits)
    for l, pr in enumerate(dw.priors):
        if len(pr.page_ids):
            ctx.kv_write(l, pr.page_ids, pr.slots, pr.k_bits, pr.v_bits)
    return ctx


def oracle_deep(dw, batch=None):
    kvs, emb = deep_oracle_pools(dw)
    b = dw.base.batch
    O.embed_txt(dw.table_bits, dw.token_ids, b.positions, emb, b.in_embed_ids)
    res = O.forward_model(dw.base.model, dw.layers, kvs, emb, batch or b, round_intermediates=True)
    return res, kvs, emb


def compare_deep(dw, what, positions_from_embeds=True):
    w, b = dw.base, dw.base.batch
    print(f"  [{what}] layers={w.model.n_layers} T={b.n_tokens} R={b.n_requests}", flush=True)
    ctx = make_deep_ctx(dw)
    ctx.embed_txt(dw.token_ids, b.positions, b.in_embed_ids)
    assert np.array_equal(ctx.embed_read(b.in_embed_ids), dw.table_bits[dw.token_ids])
    pb = ctx.batch_create(clone_batch(b, positions=None) if positions_from_embeds else b)
    ctx.forward_all(pb)
    ctx.synchronize()
    stored = np.nonzero(b.out_embed_ids >= 0)[0]
    y_bits = ctx.embed_read(b.out_embed_ids[stored])
    res, kvs, _ = oracle_deep(dw)
    assert_close(dec(y_bits), res[-1].y[stored], f"{what} output Embeds after {len(res)} layers")
    pages, slots = appended_positions(w)
    for l in range(w.model.n_layers):
        k, v = ctx.kv_read(l, pages, slots)
        # layer 0 sees bit-identical inputs; deeper layers see inputs that already differ in the last bits, so
        # only the size of a difference is bounded there, not how many values differ
        assert_bf16_close(k, res[l].k_new, f"{what} layer {l} appended K", ulps=2 if l == 0 else 4,
                          frac=0.03 if l == 0 else 1.0)
        assert_bf16_close(v, res[l].v_new, f"{what} layer {l} appended V", ulps=2 if l == 0 else 4,
                          frac=0.03 if l == 0 else 1.0)
        if len(dw.priors[l].page_ids):  # prior tokens of every layer's pool are untouched
            pk, pv = ctx.kv_read(l, dw.priors[l].page_ids, dw.priors[l].slots)
            assert np.array_equal(pk, dw.priors[l].k_bits) and np.array_equal(pv, dw.priors[l].v_bits)
    return ctx, pb, y_bits, stored


def compare_dist_deep(ctx, dw, what):
    w = dw.base
    ids = w.batch.out_embed_ids[w.dist_rows]
    gi, gp = ctx.get_next_dist(ids, w.top_k, w.temperature)
    emb = O.EmbedPool(w.n_embeds, w.model.hidden)
    emb.write(ids, ctx.embed_read(ids))  # the stored Embed is the boundary between the two calls
    oi, op, z = O.get_next_dist(w.model, w.head, emb, ids, w.top_k, w.temperature, round_intermediates=True)
    check_topk(gi, gp, z, oi, op)
    print(f"    {what}: top-{w.top_k} of {len(ids)} rows agree", flush=True)


def test_embed_txt_copies_table_rows_bit_exactly():
    dw = W.deep_tiny(n_layers=1)
    b = dw.base.batch
    ctx = make_deep_ctx(dw)
    before = ctx.embed_read(np.arange(dw.base.n_embeds))
    assert not before.any()
    ctx.embed_txt(dw.token_ids, b.positions, b.in_embed_ids)
    after = ctx.embed_read(np.arange(dw.base.n_embeds))
    _, emb = deep_oracle_pools(dw)
    O.embed_txt(dw.table_bits, dw.token_ids, b.positions, emb, b.in_embed_ids)
    assert np.array_equal(after, emb.bits)
    # ragged count, repeated tokens, last table row
    tok = np.array([dw.base.model.vocab - 1, 0, 5, 5, 5], dtype=np.int32)
    ids = np.array([95, 3, 94, 0, 17], dtype=np.int32)
    ctx.embed_txt(tok, np.arange(5), ids)
    O.embed_txt(dw.table_bits, tok, np.arange(5), emb, ids)
    assert np.array_equal(ctx.embed_read(np.arange(dw.base.n_embeds)), emb.bits)
    ctx.embed_txt([], [], [])  # empty call is a no-op


@pytest.mark.parametrize("n_layers,bitmap", [(3, False), (2, True)])
def test_deep_tiny_matches_oracle(n_layers, bitmap):
    dw = W.deep_tiny(n_layers=n_layers, bitmap=bitmap)
    ctx, *_ = compare_deep(dw, f"deep tiny L{n_layers}{' bitmap' if bitmap else ''}")
    compare_dist_deep(ctx, dw, "deep tiny dist")


def test_deep_ragged_batch_head_dim_128():
    m = W.ModelDesc(hidden=256, n_q_heads=8, n_kv_heads=2, head_dim=128, mlp_dim=384, vocab=512, page_size=16,
                    rms_eps=1e-5, rope_theta=1e4, n_layers=4)
    reqs = [W.RequestSpec(1, 0), W.RequestSpec(1, 16), W.RequestSpec(2, 100), W.RequestSpec(9, 0),
            W.RequestSpec(33, 47), W.RequestSpec(70, 130, mask=W.sink_window_mask(4, 64)),
            W.RequestSpec(1, 257, in_place=True)]
    dw = W.build_deep_workload("deep_ragged", m, reqs, n_kv_pages=96, seed=6100, std=0.05,
                               resid_std=0.05 / np.sqrt(8.0), top_k=16)
    ctx, *_ = compare_deep(dw, "deep ragged D128 L4")
    compare_dist_deep(ctx, dw, "deep ragged dist")


def test_8b_shape_two_layers_decode():
    """Two layers of the 8B shape over 16 decode requests (prior contexts 512..2048): the split-K GEMMs, the
    decode attention kernel and the wide inter-layer stream at their real widths."""
    m = W.model_8b()
    m.n_layers = 2
    ctxs = W.rng_for(6300, W.STREAM_CTX).integers(512, 2049, size=16)
    reqs = [W.RequestSpec(1, int(c), in_place=True) for c in ctxs]
    dw = W.build_deep_workload("deep_8b", m, reqs, n_kv_pages=2400, seed=6300, std=0.02,
                               resid_std=0.02 / np.sqrt(64.0), top_k=32)
    ctx, *_ = compare_deep(dw, "8B shape L2 decode")
    compare_dist_deep(ctx, dw, "8B shape L2 dist")


def test_recorded_positions_equal_explicit_positions_and_one_layer_equals_forward():
    dw = W.deep_tiny(n_layers=2)
    _, _, y_none, _ = compare_deep(dw, "positions from embed_txt", positions_from_embeds=True)
    _, _, y_expl, _ = compare_deep(dw, "explicit positions", positions_from_embeds=False)
    assert np.array_equal(y_none, y_expl)
    d1 = W.deep_tiny(n_layers=1)
    b = d1.base.batch
    ctx = make_deep_ctx(d1)
    ctx.embed_txt(d1.token_ids, b.positions, b.in_embed_ids)
    pb = ctx.batch_create(b)
    ctx.forward_all(pb)
    ctx.synchronize()
    stored = np.nonzero(b.out_embed_ids >= 0)[0]
    y_all = ctx.embed_read(b.out_embed_ids[stored])
    ctx2 = make_deep_ctx(d1)
    ctx2.embed_txt(d1.token_ids, b.positions, b.in_embed_ids)
    pb2 = ctx2.batch_create(b)
    ctx2.forward(0, pb2)
    ctx2.synchronize()
    assert np.array_equal(ctx2.embed_read(b.out_embed_ids[stored]), y_all)


def test_autoregressive_loop_follows_the_oracle():
    """The paper's prefill + decode loop (tokenised prompt, embed_txt, forward, get_next_dist, greedy pick) on
    random weights; the GPU is fed the oracle's picks so that one near-tie cannot derail the comparison."""
    m = W.model_tiny()
    m.n_layers = 2
    n_prompt, n_gen, P = 7, 6, m.page_size
    dw = W.build_deep_workload("loop", m, [W.RequestSpec(n_prompt, 0, store_all_rows=False)], n_kv_pages=8, seed=6200,
                               std=0.02, resid_std=0.02 / 2.0, top_k=8, n_embeds=16)
    prompt = dw.token_ids
    pages = dw.base.batch.page_ids[:1]  # one page holds prompt + generated tokens (13 <= 16)
    prom_emb, gen_emb = np.arange(n_prompt, dtype=np.int32), np.array([n_prompt], dtype=np.int32)
    ctx = make_deep_ctx(dw, max_batch_tokens=n_prompt)
    kvs, emb = deep_oracle_pools(dw)

    def batch(n_new, kv_len, in_ids, out_ids):
        return W.Batch(n_requests=1, n_tokens=n_new, tok_indptr=np.array([0, n_new], np.int32),
                       in_embed_ids=np.asarray(in_ids, np.int32), out_embed_ids=np.asarray(out_ids, np.int32),
                       positions=None, page_indptr=np.array([0, 1], np.int32), page_ids=pages.astype(np.int32),
                       kv_len=np.array([kv_len], np.int32))

    def step(tokens, pos, in_ids, b):
        O.embed_txt(dw.table_bits, tokens, pos, emb, in_ids)
        O.forward_model(m, dw.layers, kvs, emb, b, round_intermediates=True)
        ctx.embed_txt(tokens, pos, in_ids)
        pb = ctx.batch_create(b)
        ctx.forward_all(pb)
        ctx.synchronize()
        pb.destroy()
        got = ctx.embed_read(gen_emb)
        assert_close(dec(got), dec(emb.read(gen_emb)), "  loop output Embed")
        gi, gp = ctx.get_next_dist(gen_emb, 8, 1.0)
        probe = O.EmbedPool(16, m.hidden)
        probe.write(gen_emb, got)
        oi, op, z = O.get_next_dist(m, dw.base.head, probe, gen_emb, 8, 1.0, round_intermediates=True)
        check_topk(gi, gp, z, oi, op)
        return int(O.get_next_dist(m, dw.base.head, emb, gen_emb, 8, 1.0, round_intermediates=True)[0][0, 0])

    out_ids = np.full(n_prompt, -1, np.int32)
    out_ids[-1] = gen_emb[0]
    nxt = step(prompt, np.arange(n_prompt), prom_emb, batch(n_prompt, n_prompt, prom_emb, out_ids))
    generated = [nxt]
    for i in range(n_prompt, n_prompt + n_gen - 1):
        nxt = step([nxt], [i], gen_emb, batch(1, i + 1, gen_emb, gen_emb))
        generated.append(nxt)
    assert len(generated) == n_gen and all(0 <= t < m.vocab for t in generated)
    # the pages now hold prompt + generated tokens in every layer, equal to the oracle's within bf16 rounding
    j = np.arange(n_prompt + n_gen - 1)
    for l in range(m.n_layers):
        k, v = ctx.kv_read(l, np.full(len(j), pages[0], np.int32), j.astype(np.int32))
        ok, ov = kvs[l].read(np.full(len(j), pages[0]), j)
        assert_bf16_close(k, ok, f"loop layer {l} K", ulps=4, frac=1.0)
        assert_bf16_close(v, ov, f"loop layer {l} V", ulps=4, frac=1.0)


def test_forward_dist_equals_forward_then_get_next_dist():
    from paper_2510_24051_amd import PieError
    dw = W.deep_tiny(n_layers=2)
    w, b = dw.base, dw.base.batch
    rows = w.dist_rows
    ctx = make_deep_ctx(dw)
    ctx.embed_txt(dw.token_ids, b.positions, b.in_embed_ids)
    pb = ctx.batch_create(clone_batch(b, positions=None))
    ids1, p1 = ctx.forward_dist(pb, rows, w.top_k, 0.7)
    # against the oracle: the layer stack's output Embeds, then the distribution of the stored Embed bits
    res, _, _ = oracle_deep(dw)
    stored = np.nonzero(b.out_embed_ids >= 0)[0]
    assert_close(dec(ctx.embed_read(b.out_embed_ids[stored])), res[-1].y[stored], "forward_dist output Embeds")
    ids_e = b.out_embed_ids[rows]
    probe = O.EmbedPool(w.n_embeds, w.model.hidden)
    probe.write(ids_e, ctx.embed_read(ids_e))
    oi, op, z = O.get_next_dist(w.model, w.head, probe, ids_e, w.top_k, 0.7, round_intermediates=True)
    check_topk(ids1, p1, z / 0.7, oi, op)
    ctx2 = make_deep_ctx(dw)
    ctx2.embed_txt(dw.token_ids, b.positions, b.in_embed_ids)
    pb2 = ctx2.batch_create(clone_batch(b, positions=None))
    ctx2.forward_all(pb2)
    ids2, p2 = ctx2.get_next_dist(b.out_embed_ids[rows], w.top_k, 0.7)
    assert np.array_equal(ids1, ids2) and np.array_equal(p1, p2)
    # a row that stores no output Embed has nothing to take a distribution from; bad arguments are caught
    # before anything runs
    b3 = clone_batch(b, positions=None, out_embed_ids=b.out_embed_ids.copy())
    b3.out_embed_ids[rows[0]] = -1
    pb3 = ctx.batch_create(b3)
    for bad in (lambda: ctx.forward_dist(pb3, rows, w.top_k), lambda: ctx.forward_dist(pb, [b.n_tokens], 4),
                lambda: ctx.forward_dist(pb, rows, 0), lambda: ctx.forward_dist(pb, rows, 4, temperature=0.0)):
        with pytest.raises(PieError):
            bad()


def test_model_error_codes():
    from paper_2510_24051_amd import PieError
    dw = W.deep_tiny(n_layers=2)
    b = dw.base.batch

    def status_of(fn):
        with pytest.raises(PieError) as e:
            fn()
        return e.value.status
    ctx = make_deep_ctx(dw, load_table=False)
    assert status_of(lambda: ctx.embed_txt([1], [0], [0])) == -1           # no table loaded
    ctx.load_embedding(dw.table_bits)
    V = dw.base.model.vocab
    assert status_of(lambda: ctx.embed_txt([V], [0], [0])) == -2           # token id out of range
    assert status_of(lambda: ctx.embed_txt([-1], [0], [0])) == -2
    assert status_of(lambda: ctx.embed_txt([1], [0], [dw.base.n_embeds])) == -2
    assert status_of(lambda: ctx.embed_txt([1], [-3], [0])) == -2          # negative position
    assert status_of(lambda: ctx.embed_txt([1, 2], [0, 1], [4, 4])) == -4  # one Embed written twice
    # a batch without positions needs Embeds that carry one
    ctx.embed_write(b.in_embed_ids, dw.base.embed_bits)
    assert status_of(lambda: ctx.batch_create(clone_batch(b, positions=None))) == -1
    ctx.embed_txt(dw.token_ids, b.positions, b.in_embed_ids)
    pb = ctx.batch_create(clone_batch(b, positions=None))
    # every layer must be loaded
    from paper_2510_24051_amd import Pie
    w = dw.base
    half = Pie(w.model, w.n_kv_pages, w.n_embeds, max_batch_tokens=b.n_tokens, max_batch_requests=b.n_requests,
               max_top_k=8, max_dist_rows=1, n_layers=2)
    half.load_layer(0, dw.layers[0])
    half.embed_write(b.in_embed_ids, w.embed_bits)
    pb_half = half.batch_create(b)
    assert status_of(lambda: half.forward_all(pb_half)) == -1
    # the first context still works
    ctx.forward_all(pb)
    ctx.synchronize()
    res, _, _ = oracle_deep(dw)
    stored = np.nonzero(b.out_embed_ids >= 0)[0]
    assert_close(dec(ctx.embed_read(b.out_embed_ids[stored])), res[-1].y[stored], "after errors")
