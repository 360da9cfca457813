"""CPU pins for the oracle's KvPage control calls `mask_kvpage` and `copy_kvpage`."""
import copy

import numpy as np

import workloads as W
from oracle import pie_oracle as O
from helpers import clone_batch, oracle_pools
from test_oracle_forward import small_model, small_workload


def pages_of(b, r):
    return b.page_ids[b.page_indptr[r]:b.page_indptr[r + 1]]


def test_page_mask_equals_clearing_the_tokens_in_an_explicit_bitmap():
    w = small_workload(masks=(None, W.causal_bitmap, None))
    b, P = w.batch, w.model.page_size
    rng = np.random.default_rng(5)
    kv, emb = oracle_pools(w)
    # hide random tokens of some pages of requests 0 and 2 (prior tokens) and of request 1 (tokens it appends)
    hidden = {}
    for r in (0, 1, 2):
        for pg in pages_of(b, r)[::2]:
            hidden[int(pg)] = int(rng.integers(0, 1 << P))
    O.mask_kvpage([kv], list(hidden), list(hidden.values()))
    got = O.forward(w.model, w.weights, kv, emb, b)
    # reference: same call, no page masks, every request with an explicit bitmap that clears those tokens
    kv2, emb2 = oracle_pools(w)
    words, indptr = [], [0]
    for r in range(b.n_requests):
        n_new, L = int(b.tok_indptr[r + 1] - b.tok_indptr[r]), int(b.kv_len[r])
        allowed = W.causal_bitmap(n_new, L)
        pg = pages_of(b, r)
        for j in range(L):
            bits = hidden.get(int(pg[j // P]))
            if bits is not None and not (bits >> (j % P)) & 1:
                allowed[:, j] = False
        words.append(W.pack_mask_rows(allowed))
        indptr.append(indptr[-1] + len(words[-1]))
    ref = O.forward(w.model, w.weights, kv2, emb2,
                    clone_batch(b, mask_indptr=np.array(indptr, np.int64), mask_words=np.concatenate(words)))
    assert np.array_equal(got.y, ref.y)
    assert np.abs(got.y - O.forward(w.model, w.weights, *oracle_pools(w), b).y).max() > 1e-6  # the masks matter


def test_all_ones_page_mask_is_a_no_op_and_masks_can_be_lifted():
    w = small_workload()
    b = w.batch
    base = O.forward(w.model, w.weights, *oracle_pools(w), b)
    kv, emb = oracle_pools(w)
    O.mask_kvpage([kv], pages_of(b, 2), [0xFFFF] * len(pages_of(b, 2)))
    assert np.array_equal(O.forward(w.model, w.weights, kv, emb, b).y, base.y)
    kv, emb = oracle_pools(w)
    O.mask_kvpage([kv], pages_of(b, 2)[:1], [0x00F0])
    O.mask_kvpage([kv], pages_of(b, 2)[:1], [0xFFFF])  # the later mask replaces the earlier one
    assert np.array_equal(O.forward(w.model, w.weights, kv, emb, b).y, base.y)


def test_fully_masked_page_equals_omitted_page():
    m = small_model()
    P = m.page_size
    w = W.build_workload("drop", m, [W.RequestSpec(2, 75)], n_kv_pages=16, seed=5, std=0.2)
    b = w.batch
    kv, emb = oracle_pools(w)
    O.mask_kvpage([kv], pages_of(b, 0)[1:3], [0, 0])
    got = O.forward(w.model, w.weights, kv, emb, b)
    kv2, emb2 = oracle_pools(w)
    pages = np.concatenate([b.page_ids[:1], b.page_ids[3:]])
    short = clone_batch(b, page_ids=pages, page_indptr=np.array([0, len(pages)], np.int32),
                        kv_len=b.kv_len - 2 * P)
    ref = O.forward(w.model, w.weights, kv2, emb2, short)
    np.testing.assert_allclose(got.y, ref.y, rtol=1e-9, atol=1e-11)


def test_page_masks_hold_in_every_layer():
    m = small_model(n_layers=2)
    dw = W.build_deep_workload("deepmask", m, [W.RequestSpec(1, 40), W.RequestSpec(6, 10)], n_kv_pages=16, seed=8, std=0.2)
    from helpers import deep_oracle_pools
    b = dw.base.batch

    def run(mask_layers):
        kvs, emb = deep_oracle_pools(dw)
        O.embed_txt(dw.table_bits, dw.token_ids, b.positions, emb, b.in_embed_ids)
        if mask_layers:
            O.mask_kvpage([kvs[l] for l in mask_layers], pages_of(b, 0)[:2], [0x0F0F, 0x3333])
        return O.forward_model(m, dw.layers, kvs, emb, b)
    both, only0, none = run([0, 1]), run([0]), run([])
    assert np.array_equal(only0[0].y, both[0].y) and not np.array_equal(none[0].y, both[0].y)
    assert not np.array_equal(only0[1].y, both[1].y)  # the second layer honours the mask as well


def test_copy_kvpage_moves_bits_token_by_token_in_every_layer():
    w = small_workload()
    b, P = w.batch, w.model.page_size
    rng = np.random.default_rng(3)
    kvs = [oracle_pools(w)[0] for _ in range(3)]
    for l, kv in enumerate(kvs):  # different contents per layer
        kv.k_bits ^= np.uint16(l * 257)
    before = [(kv.k_bits.copy(), kv.v_bits.copy()) for kv in kvs]
    used = set(b.page_ids.tolist())
    spare = np.array([p for p in range(w.n_kv_pages) if p not in used][:4])
    sp = rng.choice(pages_of(b, 2), size=37)
    ss = rng.integers(0, P, size=37)
    dst = rng.permutation(4 * P)[:37]
    dp, ds = spare[dst // P], dst % P
    O.copy_kvpage(kvs, sp, ss, dp, ds)
    for kv, (k0, v0) in zip(kvs, before):
        ek, ev = k0.copy(), v0.copy()
        for a in range(37):  # hand-written slot loop
            ek[dp[a], ds[a]] = k0[sp[a], ss[a]]
            ev[dp[a], ds[a]] = v0[sp[a], ss[a]]
        assert np.array_equal(kv.k_bits, ek) and np.array_equal(kv.v_bits, ev)
        assert kv.visible.all()


def test_request_over_copied_pages_equals_request_over_the_originals():
    w = small_workload()
    b, P = w.batch, w.model.page_size
    base = O.forward(w.model, w.weights, *oracle_pools(w), b)
    kv, emb = oracle_pools(w)
    used = set(b.page_ids.tolist())
    spare = [p for p in range(w.n_kv_pages) if p not in used]
    old = pages_of(b, 2)
    new = np.array(spare[:len(old)], dtype=np.int32)
    prior = int(b.kv_len[2] - (b.tok_indptr[3] - b.tok_indptr[2]))
    j = np.arange(prior)
    O.copy_kvpage([kv], old[j // P], j % P, new[j // P], j % P)
    pages = b.page_ids.copy()
    pages[b.page_indptr[2]:b.page_indptr[3]] = new
    moved = O.forward(w.model, w.weights, kv, emb, clone_batch(b, page_ids=pages))
    assert np.array_equal(moved.y, base.y)
