"""GPU parity (through the C ABI) for the KvPage control calls `mask_kvpage` and `copy_kvpage`."""
import copy

import numpy as np
import pytest

import workloads as W
from oracle import pie_oracle as O
from helpers import clone_batch, deep_oracle_pools, oracle_pools
from gpu_helpers import assert_close, dec, gpu_forward, make_ctx
from test_gpu_model import make_deep_ctx

pytestmark = pytest.mark.gpu


def small_model(head_dim=64, n_q=4, n_kv=2):
    return W.ModelDesc(hidden=128, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=head_dim, mlp_dim=256, vocab=512,
                       page_size=16, rms_eps=1e-5, rope_theta=1e4, n_layers=1)


def random_mask(p):
    def f(n_new, L, rng):
        return (rng.random((n_new, L)) < p) & W.causal_bitmap(n_new, L)
    return f


def masked_workload(head_dim=64, n_q=4, n_kv=2, seed=900):
    m = small_model(head_dim, n_q, n_kv)
    P = 16
    reqs = [W.RequestSpec(1, 70), W.RequestSpec(1, 45, mask=W.causal_bitmap), W.RequestSpec(2, 100, mask=random_mask(0.5)),
            W.RequestSpec(40, 37), W.RequestSpec(35, 0, mask=W.causal_bitmap),
            W.RequestSpec(1, 4 * P + 3, prefix_group=0, prefix_len=4 * P),
            W.RequestSpec(1, 4 * P + 9, prefix_group=0, prefix_len=4 * P),
            W.RequestSpec(1, 4 * P + 30, prefix_group=0, prefix_len=4 * P, mask=W.causal_bitmap),
            W.RequestSpec(1, 20)]
    return W.build_workload("masked", m, reqs, n_kv_pages=96, seed=seed, std=0.05)


def pick_masks(w, seed):
    """Random token masks on every other page in use, one page fully hidden, one page that hides the tokens a
    request appends in this very call."""
    b = w.batch
    rng = np.random.default_rng(seed)
    pages = np.unique(b.page_ids)[::2]
    bits = rng.integers(0, 1 << 16, size=len(pages)).astype(np.uint32)
    bits[0] = 0
    return pages.astype(np.int32), bits


@pytest.mark.parametrize("head_dim,n_q,n_kv", [(64, 4, 2), (128, 8, 2)])
def test_page_masks_match_oracle(head_dim, n_q, n_kv):
    w = masked_workload(head_dim, n_q, n_kv)
    b = w.batch
    pages, bits = pick_masks(w, 1)
    ctx = make_ctx(w)
    ctx.mask_kvpage(pages, bits)
    pb, stored, y_bits = gpu_forward(ctx, w)
    kv, emb = oracle_pools(w)
    O.mask_kvpage([kv], pages, bits)
    res = O.forward(w.model, w.weights, kv, emb, b, round_intermediates=True)
    assert_close(dec(y_bits), res.y[stored], f"page masks D{head_dim} {n_q}/{n_kv}")
    # pages without a visible key are not visited: same count as from the oracle's own visibility rule
    P = w.model.page_size
    visited = 0
    for r in range(b.n_requests):
        n_new, L = int(b.tok_indptr[r + 1] - b.tok_indptr[r]), int(b.kv_len[r])
        pg = b.page_ids[b.page_indptr[r]:b.page_indptr[r + 1]]
        j = np.arange(L)
        if b.mask_indptr is not None and b.mask_indptr[r + 1] > b.mask_indptr[r]:
            wpr = (L + 31) // 32
            rows = [O.mask_row_bits(b.mask_words[b.mask_indptr[r] + i * wpr: b.mask_indptr[r] + (i + 1) * wpr], L)
                    for i in range(n_new)]
            allowed = np.array(rows, dtype=bool)
        else:
            allowed = W.causal_bitmap(n_new, L)
        allowed = allowed & kv.visible[pg[j // P], j % P][None, :]
        visited += len(np.unique(j[allowed.any(axis=0)] // P))
    assert pb.work()["visited_pages"] == visited
    # an unmasked run differs, and lifting the masks restores it bit for bit
    ctx0 = make_ctx(w)
    _, _, y_plain = gpu_forward(ctx0, w)
    assert not np.array_equal(y_plain, y_bits)
    ctx2 = make_ctx(w)
    ctx2.mask_kvpage(pages, bits)
    ctx2.mask_kvpage(pages, np.full(len(pages), 0xFFFF, np.uint32))
    _, _, y_lifted = gpu_forward(ctx2, w)
    assert np.array_equal(y_lifted, y_plain)


def test_page_masks_hold_in_every_layer():
    dw = W.deep_tiny(n_layers=3)
    b = dw.base.batch
    pages, bits = pick_masks(dw.base, 2)
    ctx = make_deep_ctx(dw)
    ctx.embed_txt(dw.token_ids, b.positions, b.in_embed_ids)
    ctx.mask_kvpage(pages, bits)
    pb = ctx.batch_create(clone_batch(b, positions=None))
    ctx.forward_all(pb)
    ctx.synchronize()
    stored = np.nonzero(b.out_embed_ids >= 0)[0]
    y_bits = ctx.embed_read(b.out_embed_ids[stored])
    kvs, emb = deep_oracle_pools(dw)
    O.embed_txt(dw.table_bits, dw.token_ids, b.positions, emb, b.in_embed_ids)
    O.mask_kvpage(kvs, pages, bits)
    res = O.forward_model(dw.base.model, dw.layers, kvs, emb, b, round_intermediates=True)
    assert_close(dec(y_bits), res[-1].y[stored], "page masks through 3 layers")


def test_copy_kvpage_is_bit_exact_in_every_layer_and_preserves_results():
    dw = W.deep_tiny(n_layers=2)
    w, b, P = dw.base, dw.base.batch, dw.base.model.page_size
    ctx = make_deep_ctx(dw)
    kvs, _ = deep_oracle_pools(dw)
    used = set(b.page_ids.tolist())
    spare = np.array([p for p in range(w.n_kv_pages) if p not in used], dtype=np.int32)
    # request 3 (prior 100 tokens, 7 pages): every prior token moves to a spare page, same slot
    r = 3
    old = b.page_ids[b.page_indptr[r]:b.page_indptr[r + 1]]
    new = spare[:len(old)]
    prior = int(b.kv_len[r] - 1)
    j = np.arange(prior)
    ctx.copy_kvpage(old[j // P], j % P, new[j // P], j % P)
    O.copy_kvpage(kvs, old[j // P], j % P, new[j // P], j % P)
    all_pages = np.repeat(np.arange(w.n_kv_pages, dtype=np.int32), P)
    all_slots = np.tile(np.arange(P, dtype=np.int32), w.n_kv_pages)
    for l in range(2):
        k, v = ctx.kv_read(l, all_pages, all_slots)
        assert np.array_equal(k.reshape(kvs[l].k_bits.shape), kvs[l].k_bits), f"layer {l} K"
        assert np.array_equal(v.reshape(kvs[l].v_bits.shape), kvs[l].v_bits), f"layer {l} V"
    # scattered single tokens, different slots
    rng = np.random.default_rng(4)
    sp, ss = rng.choice(old, size=11), rng.integers(0, P, size=11)
    free = rng.permutation(len(spare[len(old):]) * P)[:11]
    dp, ds = spare[len(old):][free // P], (free % P).astype(np.int32)
    ctx.copy_kvpage(sp, ss, dp, ds)
    O.copy_kvpage(kvs, sp, ss, dp, ds)
    for l in range(2):
        k, v = ctx.kv_read(l, all_pages, all_slots)
        assert np.array_equal(k.reshape(kvs[l].k_bits.shape), kvs[l].k_bits)
        assert np.array_equal(v.reshape(kvs[l].v_bits.shape), kvs[l].v_bits)
    # the request over the copied pages gives the same bits as over the originals
    ctx.embed_txt(dw.token_ids, b.positions, b.in_embed_ids)
    before = ctx.embed_read(np.arange(w.n_embeds))
    stored = np.nonzero(b.out_embed_ids >= 0)[0]
    pb = ctx.batch_create(b)
    ctx.forward_all(pb)
    ctx.synchronize()
    y0 = ctx.embed_read(b.out_embed_ids[stored])
    ctx.embed_write(np.arange(w.n_embeds), before)  # in-place requests overwrote their inputs
    ctx.embed_txt(dw.token_ids, b.positions, b.in_embed_ids)
    pages = b.page_ids.copy()
    pages[b.page_indptr[r]:b.page_indptr[r + 1]] = new
    pb2 = ctx.batch_create(clone_batch(b, page_ids=pages))
    ctx.forward_all(pb2)
    ctx.synchronize()
    assert np.array_equal(ctx.embed_read(b.out_embed_ids[stored]), y0)


def test_kvpage_error_codes():
    from paper_2510_24051_amd import PieError
    w = masked_workload()
    ctx = make_ctx(w)

    def status_of(fn):
        with pytest.raises(PieError) as e:
            fn()
        return e.value.status
    assert status_of(lambda: ctx.mask_kvpage([w.n_kv_pages], [1])) == -2
    assert status_of(lambda: ctx.mask_kvpage([-1], [1])) == -2
    assert status_of(lambda: ctx.copy_kvpage([0], [0], [w.n_kv_pages], [0])) == -2
    assert status_of(lambda: ctx.copy_kvpage([0], [16], [1], [0])) == -2
    assert status_of(lambda: ctx.copy_kvpage([0, 1], [0, 0], [2, 2], [5, 5])) == -4   # written twice
    assert status_of(lambda: ctx.copy_kvpage([0, 1], [0, 0], [1, 2], [0, 0])) == -4   # read and written
    ctx.copy_kvpage([], [], [], [])
    ctx.mask_kvpage([], [])
    _, stored, y = gpu_forward(ctx, w)  # still usable
    res = O.forward(w.model, w.weights, *oracle_pools(w), w.batch, round_intermediates=True)
    assert_close(dec(y), res.y[stored], "after errors")


# ---------------------------------------------------------------- KvPages of 32 tokens
def test_pages_of_32_tokens_forward_masks_and_copies():
    """KvPages of 32 tokens (stored as two 16-token blocks): a ragged mixed batch with bitmaps, a shared prefix,
    token-level page masks over all 32 slots and token-level copies across the two halves of a page, all against the
    oracle, which takes the page size as it is."""
    m = W.ModelDesc(hidden=128, n_q_heads=8, n_kv_heads=2, head_dim=128, mlp_dim=256, vocab=512, page_size=32,
                    rms_eps=1e-5, rope_theta=1e4, n_layers=1)
    P = 32
    reqs = [W.RequestSpec(1, 70), W.RequestSpec(1, 31), W.RequestSpec(1, 32, mask=W.causal_bitmap),
            W.RequestSpec(2, 100, mask=random_mask(0.5)), W.RequestSpec(45, 37), W.RequestSpec(35, 0, mask=W.causal_bitmap),
            W.RequestSpec(1, 2 * P + 3, prefix_group=0, prefix_len=2 * P),
            W.RequestSpec(1, 2 * P + 40, prefix_group=0, prefix_len=2 * P),
            W.RequestSpec(1, 700, mask=random_mask(0.02)), W.RequestSpec(1, 15, in_place=True)]
    w = W.build_workload("p32", m, reqs, n_kv_pages=64, seed=930, std=0.05, top_k=8)
    b = w.batch
    ctx = make_ctx(w)
    # pool round trip through (page, slot) with slots up to 31
    k0, v0 = ctx.kv_read(0, w.prior.page_ids, w.prior.slots)
    assert np.array_equal(k0, w.prior.k_bits) and np.array_equal(v0, w.prior.v_bits) and w.prior.slots.max() == 31
    rng = np.random.default_rng(5)
    pages = np.unique(b.page_ids)[::2].astype(np.int32)
    bits = rng.integers(0, 1 << 32, size=len(pages), dtype=np.uint64).astype(np.uint32)
    bits[0] = 0xFFFF0000  # the lower half of a page hidden, the upper half visible
    ctx.mask_kvpage(pages, bits)
    kv, emb = oracle_pools(w)
    O.mask_kvpage([kv], pages, bits)
    # token-level copies from a prior page into a spare one, crossing the 16-token halves
    spare = int(np.setdiff1d(np.arange(w.n_kv_pages), b.page_ids)[0])
    src_page = int(b.page_ids[0])
    ss = np.array([3, 15, 16, 31], np.int32)
    ds = np.array([16, 0, 31, 15], np.int32)
    sp, dp = np.full(4, src_page, np.int32), np.full(4, spare, np.int32)
    ctx.copy_kvpage(sp, ss, dp, ds)
    O.copy_kvpage([kv], sp, ss, dp, ds)
    gk, gv = ctx.kv_read(0, dp, ds)
    ok, ov = kv.read(dp, ds)
    assert np.array_equal(gk, ok) and np.array_equal(gv, ov)
    pb, stored, y_bits = gpu_forward(ctx, w)
    res = O.forward(m, w.weights, kv, emb, b, round_intermediates=True)
    assert_close(dec(y_bits), res.y[stored], "pages of 32 tokens: y")
    from gpu_helpers import appended_positions, assert_bf16_close
    ap, asl = appended_positions(w)
    k_gpu, v_gpu = ctx.kv_read(0, ap, asl)
    assert_bf16_close(k_gpu, res.k_new, "pages of 32 tokens: appended K", ulps=2)
    assert_bf16_close(v_gpu, res.v_new, "pages of 32 tokens: appended V", ulps=2)
    # the shared prefix is still read once for both requests
    work = pb.work()
    assert work["kv_bytes_requested"] < work["kv_bytes_decode"]
    ctx.close()
