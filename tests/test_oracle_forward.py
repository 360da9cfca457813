"""CPU pins for the oracle's `forward` / `get_next_dist` handlers: invariants the paper states for
the calls, plus an independent torch CPU expression of a textbook Llama decoder layer."""
import copy

import numpy as np
import torch
import torch.nn.functional as F

import workloads as W
from oracle import pie_oracle as O
from helpers import clone_batch, oracle_pools, run_oracle

TOL = dict(rtol=1e-9, atol=1e-11)


def small_model(page_size=16, **kw):
    d = dict(hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16, mlp_dim=96, vocab=200, page_size=page_size,
             rms_eps=1e-5, rope_theta=1e4, n_layers=1)
    d.update(kw)
    return W.ModelDesc(**d)


def small_workload(seed=11, page_size=16, masks=(None, None, None), std=0.2, **kw):
    m = small_model(page_size)
    reqs = [W.RequestSpec(1, 21, mask=masks[0]), W.RequestSpec(9, 0, mask=masks[1]),
            W.RequestSpec(5, 30, mask=masks[2])]
    return W.build_workload("small", m, reqs, n_kv_pages=(64 * 16) // page_size, seed=seed, std=std, top_k=5, **kw)


def dec(bits):
    return O.bf16_decode(bits)


# ---------------------------------------------------------------- whole layer against torch CPU
def torch_llama_layer(model, w, x, pos, act_bf16=False, taps=None):
    """Textbook pre-norm Llama layer for ONE contiguous causal sequence, written with torch library ops.
    `act_bf16`: cast to torch.bfloat16 (and back) exactly where the paper's stated activation precision puts a
    bf16 tensor between two contractions: the normalised input, q/k/v as projected, q after the rotary step, the
    attention output, the second norm's output and the SwiGLU product; the residual stream stays wide."""
    H, Hq, Hkv, D = model.hidden, model.n_q_heads, model.n_kv_heads, model.head_dim
    t = lambda b: torch.from_numpy(dec(b))
    r = (lambda a: a.to(torch.bfloat16).to(torch.float64)) if act_bf16 else (lambda a: a)
    xn = r(F.rms_norm(x, (H,), t(w.g1), eps=model.rms_eps))
    q = r(F.linear(xn, t(w.wq))).view(-1, Hq, D)
    k = r(F.linear(xn, t(w.wk))).view(-1, Hkv, D)
    v = r(F.linear(xn, t(w.wv))).view(-1, Hkv, D)

    def rot(a):  # complex formulation of the rotary step
        z = torch.complex(a[..., : D // 2], a[..., D // 2:])
        freq = model.rope_theta ** (-torch.arange(0, D, 2, dtype=torch.float64) / D)
        ph = torch.polar(torch.ones_like(pos[:, None] * freq), pos[:, None] * freq)[:, None, :]
        z = z * ph
        return torch.cat([z.real, z.imag], dim=-1)

    q, k = r(rot(q)), rot(k)
    k = k.to(torch.bfloat16).to(torch.float64)  # KvPages are bf16 storage
    v = v.to(torch.float32).to(torch.bfloat16).to(torch.float64)
    g = Hq // Hkv
    o = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], k.permute(1, 0, 2).repeat_interleave(g, 0)[None],
                                       v.permute(1, 0, 2).repeat_interleave(g, 0)[None], is_causal=True)
    o = r(o[0].permute(1, 0, 2).reshape(-1, Hq * D))
    h = x + F.linear(o, t(w.wo))
    hn = r(F.rms_norm(h, (H,), t(w.g2), eps=model.rms_eps))
    act = r(F.silu(F.linear(hn, t(w.wgate))) * F.linear(hn, t(w.wup)))
    if taps is not None:
        taps.update(q=q, o=o, h=h, act=act)
    return h + F.linear(act, t(w.wdown))


def test_layer_matches_torch_textbook_layer():
    m = small_model()
    wl = W.build_workload("one", m, [W.RequestSpec(23, 0)], n_kv_pages=8, seed=3, std=0.2)
    res, kv, emb = run_oracle(wl)
    x = torch.from_numpy(dec(wl.embed_bits))
    pos = torch.from_numpy(wl.batch.positions.astype(np.float64))
    ref = torch_llama_layer(m, wl.weights, x, pos).numpy()
    # torch casts k through float32->bf16 (double rounding is possible but rare); allow bf16-level slack on few
    np.testing.assert_allclose(res.y, ref, rtol=1e-6, atol=2e-3)
    assert np.mean(np.abs(res.y - ref)) < 1e-5
    # stored Embeds are the bf16 rounding of y
    got = dec(emb.read(wl.batch.out_embed_ids))
    assert np.array_equal(got, O.bf16_round(res.y))


def test_zero_residual_projections_give_identity():
    wl = small_workload()
    wl.weights.wo[:] = 0
    wl.weights.wdown[:] = 0
    res, _, _ = run_oracle(wl)
    assert np.array_equal(res.y, dec(wl.embed_bits))


# ---------------------------------------------------------------- masks
def test_explicit_causal_bitmap_equals_inferred():
    a, _, _ = run_oracle(small_workload())
    b, _, _ = run_oracle(small_workload(masks=(W.causal_bitmap,) * 3))
    assert np.array_equal(a.y, b.y)
    # mixed: only one request carries a bitmap, the others are inferred
    c, _, _ = run_oracle(small_workload(masks=(None, W.causal_bitmap, None)))
    assert np.array_equal(a.y, c.y)


def test_masking_whole_pages_equals_omitting_them():
    """Forward API: leaving out the KvPage of earlier tokens masks those tokens."""
    m = small_model()
    P = m.page_size

    def hide_pages(n_new, L, rng):
        a = W.causal_bitmap(n_new, L)
        a[:, P:3 * P] = False  # pages 1 and 2 of the request hidden
        return a

    full = W.build_workload("hide", m, [W.RequestSpec(2, 75, mask=hide_pages)], n_kv_pages=16, seed=5, std=0.2)
    res_full, kv_full, _ = run_oracle(full)
    # same request with pages 1,2 dropped from the table: logical length shrinks by 2P, positions unchanged
    b = full.batch
    pages = np.concatenate([b.page_ids[:1], b.page_ids[3:]])
    nb = clone_batch(b, page_ids=pages, page_indptr=np.array([0, len(pages)], np.int32),
                     kv_len=b.kv_len - 2 * P, mask_indptr=None, mask_words=None)
    kv, emb = oracle_pools(full)
    res_drop = O.forward(m, full.weights, kv, emb, nb)
    np.testing.assert_allclose(res_drop.y, res_full.y, **TOL)


# ---------------------------------------------------------------- page table
def test_page_id_permutation_invariance():
    a = small_workload(seed=11)
    res_a, _, _ = run_oracle(a)
    perm = np.random.default_rng(0).permutation(a.n_kv_pages).astype(np.int32)
    b = copy.deepcopy(a)
    b.batch.page_ids = perm[a.batch.page_ids]
    b.prior.page_ids = perm[a.prior.page_ids]
    res_b, _, _ = run_oracle(b)
    assert np.array_equal(res_a.y, res_b.y)


def test_page_size_1_vs_16():
    a = small_workload(page_size=16)
    b = small_workload(page_size=1)
    # same tokens, same draws (prior KV is drawn per token in request order in both layouts)
    assert np.array_equal(a.prior.k_bits, b.prior.k_bits) and np.array_equal(a.embed_bits, b.embed_bits)
    res_a, _, _ = run_oracle(a)
    res_b, _, _ = run_oracle(b)
    assert np.array_equal(res_a.y, res_b.y)


def test_aliased_pages_equal_private_copies():
    m = small_model()
    shared = [W.RequestSpec(1, 32 + 7, prefix_group=0, prefix_len=32) for _ in range(3)]
    a = W.build_workload("alias", m, shared, n_kv_pages=32, seed=9, std=0.2)
    res_a, kv_a, _ = run_oracle(a)
    # private copies: give every request its own pages and copy the prefix tokens into them
    b = copy.deepcopy(a)
    P = m.page_size
    used = set(a.batch.page_ids.tolist())
    spare = [p for p in range(a.n_kv_pages) if p not in used]
    kv_b, emb_b = oracle_pools(a)
    pages = b.batch.page_ids.copy()
    for r in (1, 2):
        for i in range(32 // P):
            idx = b.batch.page_indptr[r] + i
            new = spare.pop()
            kv_b.k_bits[new] = kv_b.k_bits[pages[idx]]
            kv_b.v_bits[new] = kv_b.v_bits[pages[idx]]
            pages[idx] = new
    b.batch.page_ids = pages
    assert len(set(pages.tolist())) == len(pages)
    res_b = O.forward(m, b.weights, kv_b, emb_b, b.batch)
    assert np.array_equal(res_a.y, res_b.y)
    # distinct suffixes -> branches differ from each other
    assert not np.array_equal(res_a.y[0], res_a.y[1])


# ---------------------------------------------------------------- append and split calls
def test_split_call_equivalence():
    """Forward API example: one call over 9 tokens == a call over 8 tokens that only fills KvPages,
    then a call over the 9th token that reads them."""
    m = small_model()
    one = W.build_workload("split", m, [W.RequestSpec(9, 0)], n_kv_pages=4, seed=21, std=0.2)
    res_one, kv_one, _ = run_oracle(one)
    b = one.batch
    kv, emb = oracle_pools(one)
    first = clone_batch(b, n_tokens=8, tok_indptr=np.array([0, 8], np.int32), in_embed_ids=b.in_embed_ids[:8],
                        out_embed_ids=np.full(8, -1, np.int32), positions=b.positions[:8],
                        kv_len=np.array([8], np.int32))
    O.forward(m, one.weights, kv, emb, first)
    second = clone_batch(b, n_tokens=1, tok_indptr=np.array([0, 1], np.int32), in_embed_ids=b.in_embed_ids[8:],
                         out_embed_ids=b.out_embed_ids[8:], positions=b.positions[8:],
                         kv_len=np.array([9], np.int32))
    res_two = O.forward(m, one.weights, kv, emb, second)
    np.testing.assert_allclose(res_two.y[0], res_one.y[8], **TOL)
    assert np.array_equal(kv.k_bits, kv_one.k_bits) and np.array_equal(kv.v_bits, kv_one.v_bits)


def test_append_lands_in_the_right_slot_and_leaves_the_rest():
    wl = small_workload()
    kv0, _ = oracle_pools(wl)
    res, kv, _ = run_oracle(wl)
    b, P = wl.batch, wl.model.page_size
    touched = np.zeros(kv.k_bits.shape[:2], dtype=bool)
    for r in range(b.n_requests):
        n_new = b.tok_indptr[r + 1] - b.tok_indptr[r]
        pages = b.page_ids[b.page_indptr[r]:b.page_indptr[r + 1]]
        for i in range(n_new):
            j = b.kv_len[r] - n_new + i
            t = b.tok_indptr[r] + i
            assert np.array_equal(kv.k_bits[pages[j // P], j % P], res.k_new[t])
            assert np.array_equal(kv.v_bits[pages[j // P], j % P], res.v_new[t])
            touched[pages[j // P], j % P] = True
    assert np.array_equal(kv.k_bits[~touched], kv0.k_bits[~touched])


def test_rope_shift_invariance_without_prior_context():
    m = small_model()
    wl = W.build_workload("shift", m, [W.RequestSpec(12, 0)], n_kv_pages=4, seed=2, std=0.2)
    res_a, _, _ = run_oracle(wl)
    wl2 = copy.deepcopy(wl)
    wl2.batch.positions = wl.batch.positions + 1000
    res_b, _, _ = run_oracle(wl2)
    # K pages are rounded to bf16 after rotation, so equality holds to bf16-level effects on the scores only
    assert np.abs(res_a.y - res_b.y).max() < 0.02 * np.abs(res_a.y).max()
    assert np.abs(res_a.y - res_b.y).mean() < 0.003 * np.abs(res_a.y).mean()
    assert not np.array_equal(res_a.k_new, res_b.k_new)


def test_positions_are_independent_of_storage_slot():
    """Explicit positions drive the rotary step; the logical index drives storage and causality."""
    wl = small_workload()
    res_a, kv_a, _ = run_oracle(wl)
    wl2 = copy.deepcopy(wl)
    wl2.batch.positions = wl.batch.positions + 7
    res_b, kv_b, _ = run_oracle(wl2)
    assert np.array_equal(kv_a.v_bits, kv_b.v_bits)      # V untouched by positions
    assert not np.array_equal(kv_a.k_bits, kv_b.k_bits)  # K rotated differently, same slots
    assert np.array_equal((kv_a.k_bits != 0).any(axis=(2, 3)), (kv_b.k_bits != 0).any(axis=(2, 3)))


# ---------------------------------------------------------------- batching
def test_batch_composition_and_order_invariance():
    wl = small_workload()
    res, _, _ = run_oracle(wl)
    b = wl.batch
    # each request alone
    for r in range(b.n_requests):
        a, e = b.tok_indptr[r], b.tok_indptr[r + 1]
        pa, pe = b.page_indptr[r], b.page_indptr[r + 1]
        solo = clone_batch(b, n_requests=1, n_tokens=e - a, tok_indptr=np.array([0, e - a], np.int32),
                           in_embed_ids=b.in_embed_ids[a:e], out_embed_ids=b.out_embed_ids[a:e],
                           positions=b.positions[a:e], page_indptr=np.array([0, pe - pa], np.int32),
                           page_ids=b.page_ids[pa:pe], kv_len=b.kv_len[r:r + 1])
        kv, emb = oracle_pools(wl)
        rs = O.forward(wl.model, wl.weights, kv, emb, solo)
        np.testing.assert_allclose(rs.y, res.y[a:e], **TOL)
    # reversed request order
    order = [2, 1, 0]
    toks = np.concatenate([np.arange(b.tok_indptr[r], b.tok_indptr[r + 1]) for r in order])
    pgs = np.concatenate([b.page_ids[b.page_indptr[r]:b.page_indptr[r + 1]] for r in order])
    n_tok = np.array([b.tok_indptr[r + 1] - b.tok_indptr[r] for r in order])
    n_pg = np.array([b.page_indptr[r + 1] - b.page_indptr[r] for r in order])
    rev = clone_batch(b, tok_indptr=np.concatenate([[0], np.cumsum(n_tok)]).astype(np.int32),
                      in_embed_ids=b.in_embed_ids[toks], out_embed_ids=b.out_embed_ids[toks],
                      positions=b.positions[toks], page_ids=pgs,
                      page_indptr=np.concatenate([[0], np.cumsum(n_pg)]).astype(np.int32), kv_len=b.kv_len[order])
    kv, emb = oracle_pools(wl)
    rr = O.forward(wl.model, wl.weights, kv, emb, rev)
    np.testing.assert_allclose(rr.y, res.y[toks], **TOL)


def test_rows_subset_and_unstored_rows():
    wl = small_workload()
    full, _, emb_full = run_oracle(wl)
    rows = np.array([0, 4, 9, 14])
    part, _, _ = run_oracle(wl, rows=rows)
    np.testing.assert_allclose(part.y, full.y[rows], **TOL)  # BLAS blocking differs with the row count
    wl2 = copy.deepcopy(wl)
    wl2.batch.out_embed_ids[1:9] = -1  # prefill request stores only its last token
    _, _, emb2 = run_oracle(wl2)
    keep = wl.batch.out_embed_ids[[0] + list(range(9, 15))]
    assert np.array_equal(emb2.read(keep), emb_full.read(keep))
    dropped = wl.batch.out_embed_ids[1:9]
    assert not emb2.read(dropped).any()


def test_in_place_embed_is_read_before_written():
    m = small_model()
    wl = W.build_workload("inplace", m, [W.RequestSpec(3, 5, in_place=True)], n_kv_pages=4, seed=8, std=0.2)
    assert np.array_equal(wl.batch.in_embed_ids, wl.batch.out_embed_ids)
    res, _, emb = run_oracle(wl)
    wl2 = copy.deepcopy(wl)
    wl2.batch.out_embed_ids = np.array([90, 91, 92], np.int32)
    wl2.n_embeds = 100
    wl.n_embeds = 100
    res2, _, emb2 = run_oracle(wl2)
    assert np.array_equal(res.y, res2.y)
    assert np.array_equal(emb.read(wl.batch.out_embed_ids), emb2.read([90, 91, 92]))


def test_round_intermediates_mode_matches_torch_layer_with_bf16_casts():
    """The oracle's bf16-intermediate mode (the primary comparator of the GPU parity tests) against an independent
    torch expression that casts `.to(torch.bfloat16)` at exactly the points where the oracle rounds.  A rounding
    point that is missing, misplaced or added (e.g. a rounded residual stream) moves most elements of y by a bf16
    ulp of some intermediate, far above the limits here; torch's float64 -> float32 -> bf16 cast may double-round
    one value in ~2**29, which at most shows as an isolated element."""
    m = small_model(hidden=128, mlp_dim=192)
    wl = W.build_workload("one_b", m, [W.RequestSpec(37, 0)], n_kv_pages=8, seed=5, std=0.2)
    res, kv, _ = run_oracle(wl, round_intermediates=True)
    x = torch.from_numpy(dec(wl.embed_bits))
    pos = torch.from_numpy(wl.batch.positions.astype(np.float64))
    taps = {}
    ref = torch_llama_layer(m, wl.weights, x, pos, act_bf16=True, taps=taps).numpy()
    for name, got, want in (("q", res.q, taps["q"].numpy()), ("o", res.o.reshape(37, -1), taps["o"].numpy()),
                            ("h", res.h, taps["h"].numpy()), ("act", res.act, taps["act"].numpy()), ("y", res.y, ref)):
        d = np.abs(got.reshape(want.shape) - want)
        assert np.mean(d > 1e-9) < 1e-3 and d.mean() < 1e-6, (name, float(d.max()), float(d.mean()))
    # the planted alternatives are all far away: wide mode, and a torch layer that also rounds the residual stream
    wide, _, _ = run_oracle(wl)
    assert np.abs(wide.y - ref).mean() > 1e-4
    h_rounded = taps["h"].to(torch.bfloat16).to(torch.float64).numpy()
    assert np.abs(h_rounded - res.h).mean() > 1e-4  # the oracle's residual stream is not rounded
    # the head: the normalised Embed is rounded to bf16 before the LM head, the logits stay wide
    wl2 = W.c1_tiny()
    _, _, emb = run_oracle(wl2, round_intermediates=True)
    ids_e = wl2.batch.out_embed_ids[wl2.dist_rows]
    z = O.logits_from_embeds(wl2.model, wl2.head, emb, ids_e, round_intermediates=True)
    e = torch.from_numpy(dec(emb.read(ids_e)))
    en = F.rms_norm(e, (wl2.model.hidden,), torch.from_numpy(dec(wl2.head.g_final)), eps=wl2.model.rms_eps)
    zz = F.linear(en.to(torch.bfloat16).to(torch.float64), torch.from_numpy(dec(wl2.head.w_lm))).numpy()
    dz = np.abs(z - zz)
    assert np.mean(dz > 1e-9) < 1e-3 and dz.mean() < 1e-6
    z_wide = O.logits_from_embeds(wl2.model, wl2.head, emb, ids_e)
    assert np.abs(z_wide - zz).mean() > 1e-5


def test_round_intermediates_mode_is_close_to_wide_mode():
    wl = W.c1_tiny()
    a, _, _ = run_oracle(wl)
    b, _, _ = run_oracle(wl, round_intermediates=True)
    d = np.abs(a.y - b.y)
    assert 0 < d.max() < 2e-2 and d.mean() < 1e-3


# ---------------------------------------------------------------- get_next_dist
def test_get_next_dist_on_stored_embeds():
    wl = W.c1_tiny()
    res, _, emb = run_oracle(wl)
    ids_e = wl.batch.out_embed_ids[wl.dist_rows]
    ids, probs, z = O.get_next_dist(wl.model, wl.head, emb, ids_e, wl.top_k, 1.0)
    assert ids.shape == (5, 8) and np.all(np.diff(probs, axis=1) <= 0)
    # independent torch expression on the same stored bits
    e = torch.from_numpy(dec(emb.read(ids_e)))
    en = F.rms_norm(e, (wl.model.hidden,), torch.from_numpy(dec(wl.head.g_final)), eps=wl.model.rms_eps)
    zz = F.linear(en, torch.from_numpy(dec(wl.head.w_lm)))
    tv, ti = torch.topk(torch.softmax(zz, -1), 8, dim=-1)
    assert np.array_equal(ids, ti.numpy())
    np.testing.assert_allclose(probs, tv.numpy(), rtol=1e-10)
    # without a final-norm gain the norm is skipped
    head2 = W.HeadWeights(None, wl.head.w_lm)
    _, _, z2 = O.get_next_dist(wl.model, head2, emb, ids_e, 8)
    np.testing.assert_allclose(z2, F.linear(e, torch.from_numpy(dec(wl.head.w_lm))).numpy(), rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------- workload recipes (shape checks)
def test_named_workloads_scaled_down_are_consistent():
    m = small_model(head_dim=16)
    c4 = W.c4_prefix_tree(n_branches=8, prefix_len=64, suffix_prior=15, span=32, n_kv_pages=64, model=m)
    b = c4.batch
    assert b.n_requests == 8 and np.all(b.kv_len == 80) and np.all(np.diff(b.page_indptr) == 5)
    tables = b.page_ids.reshape(8, 5)
    assert np.all(tables[:, :4] == tables[0, :4]) and len(set(tables[:, 4].tolist())) == 8
    words = b.mask_words.reshape(8, 3)
    n_hidden = sum(int(bin(int(w[0]) | int(w[1]) << 32 | int(w[2]) << 64).count("1")) == 80 - 32 for w in words)
    assert n_hidden == 2  # exactly 25% of the branches hide a span
    c5 = W.c5_sparse_long(n_requests=2, ctx=300, n_sink=4, window=64, n_kv_pages=64, model=m)
    row = O.mask_row_bits(c5.batch.mask_words[: (301 + 31) // 32], 301)
    assert row[:4].all() and row[301 - 64:].all() and not row[4:301 - 64].any()
    res, _, _ = run_oracle(c4)
    assert np.isfinite(res.y).all()
