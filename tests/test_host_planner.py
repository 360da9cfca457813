"""Host logic of the library without a GPU: batch deserialisation, its error codes and the attention launch plan,
through a planner context (pie_create_planner makes no HIP call)."""
import copy
import numpy as np
import pytest

import workloads as W
from helpers import clone_batch
from paper_2510_24051_amd import Pie, PieError


def small_model(head_dim=64, n_q=4, n_kv=2, hidden=128, mlp=256):
    return W.ModelDesc(hidden=hidden, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=head_dim, mlp_dim=mlp, vocab=512,
                       page_size=16, rms_eps=1e-5, rope_theta=1e4, n_layers=1)


def random_mask(p):
    def f(n_new, L, rng):
        m = rng.random((n_new, L)) < p
        m &= W.causal_bitmap(n_new, L)
        return m
    return f


def planner_for(w, wave_slots=2048, **kw):
    b = w.batch
    return Pie.planner(w.model, w.n_kv_pages, w.n_embeds, max_batch_tokens=int(b.n_tokens),
                       max_batch_requests=int(b.n_requests), wave_slots=wave_slots, **kw)


def expected_work(w, page_mask=None):
    """The statistics of pie_batch_work recomputed from the batch description alone."""
    m, b = w.model, w.batch
    P, G = m.page_size, m.n_q_heads // m.n_kv_heads
    page_bytes = m.n_kv_heads * 2 * P * m.head_dim * 2
    visited = visited_dec = 0
    flops = 0
    distinct = set()
    n_items = n_dec = rows_cap = 0
    for r in range(b.n_requests):
        t0, t1 = int(b.tok_indptr[r]), int(b.tok_indptr[r + 1])
        n_new, L = t1 - t0, int(b.kv_len[r])
        n_pages = (L + P - 1) // P
        pages = b.page_ids[b.page_indptr[r]:b.page_indptr[r] + n_pages]
        has_mask = b.mask_indptr is not None and b.mask_indptr[r + 1] > b.mask_indptr[r]
        masked_pages = page_mask is not None and any(page_mask.get(int(p), 0xFFFF) != 0xFFFF for p in pages)
        if has_mask or masked_pages:
            if has_mask:
                wpr = (L + 31) // 32
                words = b.mask_words[b.mask_indptr[r]:b.mask_indptr[r + 1]].reshape(n_new, wpr)
                allowed = ((words[:, :, None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(n_new, wpr * 32)[:, :L].astype(bool)
            else:
                allowed = W.causal_bitmap(n_new, L)
            if masked_pages:
                vis = np.concatenate([[(page_mask.get(int(p), 0xFFFF) >> s) & 1 for s in range(P)] for p in pages])[:L].astype(bool)
                allowed = allowed & vis[None, :]
            any_key = allowed.any(axis=0)
            vis_pages = [pg for pg in range(n_pages) if any_key[pg * P:(pg + 1) * P].any()]
            explicit = True
        else:
            vis_pages, explicit = list(range(n_pages)), False
        nv = len(vis_pages)
        visited += nv
        if n_new * G <= 16:
            n_dec += 1
            rows_cap = max(rows_cap, n_new * G)
            visited_dec += nv
            distinct.update(int(pages[pg]) for pg in vis_pages)
            flops += nv * P * n_new * m.n_q_heads * m.head_dim * 4
        else:
            n_items += (n_new + 31) // 32
            if explicit:
                flops += nv * P * n_new * m.n_q_heads * m.head_dim * 4
            else:
                flops += m.n_q_heads * m.head_dim * 4 * (n_new * (L - n_new) + n_new * (n_new + 1) // 2)
    return dict(kv_bytes=visited * page_bytes, kv_bytes_decode=visited_dec * page_bytes, attn_flops=flops,
                visited_pages=visited, kv_bytes_unique=len(distinct) * page_bytes), \
        dict(prefill_items=n_items, decode_requests=n_dec, rows_cap=rows_cap)


def workloads():
    sparse = random_mask(0.3)
    yield "c1", W.c1_tiny()
    m = small_model(64, 4, 2)
    reqs = [W.RequestSpec(1, 0), W.RequestSpec(1, 15), W.RequestSpec(2, 100), W.RequestSpec(3, 33, mask=sparse),
            W.RequestSpec(9, 0), W.RequestSpec(31, 5, mask=W.causal_bitmap), W.RequestSpec(33, 47),
            W.RequestSpec(70, 130, mask=sparse), W.RequestSpec(1, 700, mask=random_mask(0.02)),
            W.RequestSpec(1, 257, in_place=True), W.RequestSpec(40, 0, mask=random_mask(0.9))]
    yield "ragged", W.build_workload("ragged", m, reqs, n_kv_pages=160, seed=100, std=0.05, with_head=False)
    P = 16
    reqs = [W.RequestSpec(1, 5 * P + 3, prefix_group=0, prefix_len=5 * P),
            W.RequestSpec(1, 5 * P + 40, prefix_group=0, prefix_len=5 * P),
            W.RequestSpec(1, 5 * P, prefix_group=0, prefix_len=5 * P, in_place=True),
            W.RequestSpec(1, 9 * P + 1, prefix_group=0, prefix_len=5 * P, mask=W.causal_bitmap),
            W.RequestSpec(1, 33), W.RequestSpec(2, 3 * P + 5, prefix_group=1, prefix_len=3 * P),
            W.RequestSpec(2, 3 * P + 20, prefix_group=1, prefix_len=3 * P),
            W.RequestSpec(40, 3 * P, prefix_group=1, prefix_len=3 * P)]
    yield "shared", W.build_workload("shared", small_model(128, 8, 2), reqs, n_kv_pages=96, seed=700, std=0.05,
                                     with_head=False)
    rng = np.random.default_rng(5)
    reqs = [W.RequestSpec(1, int(c)) for c in rng.integers(512, 4097, size=64)]
    yield "decode64", W.build_workload("decode64", small_model(64, 8, 2), reqs, n_kv_pages=12000, seed=2000, std=0.02,
                                       with_head=False)


@pytest.mark.parametrize("name,w", list(workloads()), ids=lambda x: x if isinstance(x, str) else "")
def test_plan_statistics_match_the_batch(name, w):
    ctx = planner_for(w)
    pb = ctx.batch_create(w.batch, validate=True)
    work, info = pb.work(), pb.plan_info()
    exp_work, exp_info = expected_work(w)
    for k, v in exp_work.items():
        assert work[k] == v, (name, k, work[k], v)
    for k in ("prefill_items", "decode_requests"):
        assert info[k] == exp_info[k], (name, k, info[k], exp_info[k])
    assert exp_info["rows_cap"] <= info["rows_cap"] <= 16  # wider when requests that share pages form one column group
    # requests that share pages are walked together: never more bytes than the per-request count, never fewer
    # than the distinct pages; without sharing all three agree
    assert work["kv_bytes_unique"] <= work["kv_bytes_requested"] <= work["kv_bytes_decode"]
    if name != "shared":
        assert work["kv_bytes_requested"] == work["kv_bytes_decode"] == work["kv_bytes_unique"]
    else:
        assert work["kv_bytes_requested"] < work["kv_bytes_decode"]
    assert 1 <= info["max_pairs_per_wave"] <= 64
    # every share is sized for the resident waves: the wave count is a whole number of rounds or less than one
    assert info["decode_waves"] <= 2048 or info["decode_waves"] % 2048 == 0 or info["max_pairs_per_wave"] == 64
    assert info["segments"] >= info["decode_waves"] or info["decode_waves"] == 0
    pb.destroy()
    ctx.close()


def prefill_mix(n_kv=8, sizes=((1024, 0), (1024, 1500), (512, 100), (300, 2040), (40, 0), (33, 700))):
    m = small_model(128, 4 * n_kv if n_kv <= 2 else 2 * n_kv, n_kv)
    reqs = [W.RequestSpec(n, prior) for n, prior in sizes] + [W.RequestSpec(1, 900), W.RequestSpec(1, 64)]
    pages = sum((n + p + 15) // 16 for n, p in sizes) + 80
    return W.build_workload("prefill_mix", m, reqs, n_kv_pages=pages, seed=4100 + n_kv, std=0.02, with_head=False)


@pytest.mark.parametrize("n_kv", [8, 2, 1])
def test_prefill_launch_covers_every_block_once_and_keeps_a_head_on_one_xcd(n_kv):
    """The two prefill launches together list one workgroup per (request, 32-token query block, kv head): each
    exactly once, empty slots only as padding, workgroup i of a launch on XCD i % 8; the second launch holds exactly
    the blocks whose rows may see few keys (here: causal blocks that start within the first 64 keys); within a launch
    the query blocks of one (request, kv head) share an XCD unless the planner had to cut groups to even out the
    XCDs; the XCDs' loads are even."""
    w = prefill_mix(n_kv)
    b, m = w.batch, w.model
    ctx = planner_for(w)
    pb = ctx.batch_create(w.batch, validate=True)
    work = pb.prefill_work()
    G = m.n_q_heads // m.n_kv_heads
    expected = set()
    cost = {}
    for r in range(b.n_requests):
        n_new = int(b.tok_indptr[r + 1] - b.tok_indptr[r])
        if n_new * G <= 16:
            continue
        for qb in range((n_new + 31) // 32):
            for hk in range(m.n_kv_heads):
                expected.add((r, qb, hk))
                cost[(r, qb, hk)] = int(b.kv_len[r]) - n_new + min(n_new, qb * 32 + 32)
    assert pb.plan_info()["prefill_items"] * m.n_kv_heads == len(expected)
    info = pb.plan_info()
    n_plain, n_pair = info["prefill_workgroups"], info["prefill_workgroups_pair_weights"]
    assert work.shape[0] == n_plain + n_pair and n_plain % 8 == 0 and n_pair % 8 == 0
    real = [tuple(int(x) for x in row) for row in work if row[0] >= 0]
    assert len(real) == len(set(real)) == len(expected) and set(real) == expected
    assert all(row[1] == 0 and row[2] == 0 for row in work if row[0] < 0)
    few = lambda r, qb: int(b.kv_len[r]) - int(b.tok_indptr[r + 1] - b.tok_indptr[r]) + qb * 32 < 64
    assert {k for k in map(tuple, work[n_plain:].tolist()) if k[0] >= 0} == {k for k in expected if few(k[0], k[1])}
    assert n_pair > 0
    work_all, work = work, work[:n_plain]  # the layout properties below are those of one launch: the large one
    xcd_of, load = {}, np.zeros(8)
    for i, row in enumerate(work):
        if row[0] >= 0:
            key = (int(row[0]), int(row[1]), int(row[2]))
            xcd_of.setdefault((key[0], key[2]), set()).add(i % 8)
            load[i % 8] += cost[key]
    groups = len(xcd_of)
    if groups >= 16:  # enough groups to balance whole: none is cut
        assert all(len(v) == 1 for v in xcd_of.values())
    # even loads: no XCD more than a quarter above the mean, unless a single query block is that heavy
    heaviest = max(cost.values())
    assert load.max() <= max(1.25 * load.mean(), load.mean() + heaviest), load
    # within an XCD's list the blocks of a group are next to each other when groups are whole
    if groups >= 16:
        for x in range(8):
            seq = [(int(r), int(h)) for r, q, h in work[x::8] if r >= 0]
            changes = sum(1 for a, c in zip(seq, seq[1:]) if a != c)
            assert changes == len(set(seq)) - 1
    # the accessor copies at most `cap` entries and always reports the total; bad arguments are refused
    import ctypes as C
    n = C.c_int32(0)
    part = np.full((5, 3), -7, dtype=np.int32)
    assert ctx.lib.pie_batch_prefill_work(pb.handle, part.ctypes.data_as(C.c_void_p), 5, C.byref(n)) == 0
    assert n.value == work_all.shape[0] and (part == work_all[:5]).all()
    assert ctx.lib.pie_batch_prefill_work(pb.handle, None, 3, C.byref(n)) == -1
    assert ctx.lib.pie_batch_prefill_work(pb.handle, part.ctypes.data_as(C.c_void_p), 5, None) == -1
    assert ctx.lib.pie_batch_prefill_work(None, part.ctypes.data_as(C.c_void_p), 5, C.byref(n)) == -1
    pb.destroy()
    ctx.close()


def test_plan_depends_on_the_resident_waves_but_the_work_does_not():
    w = dict(workloads())["decode64"]
    small, big = planner_for(w, wave_slots=64), planner_for(w, wave_slots=2048)
    a, b = small.batch_create(w.batch), big.batch_create(w.batch)
    assert a.work() == b.work()
    ia, ib = a.plan_info(), b.plan_info()
    assert ia["decode_waves"] < ib["decode_waves"] and ia["max_pairs_per_wave"] > ib["max_pairs_per_wave"]
    pairs = sum((int(L) + 31) // 32 for L in w.batch.kv_len) * w.model.n_kv_heads
    for info in (ia, ib):  # the shares cover every (request, kv head, page pair)
        assert info["decode_waves"] * info["max_pairs_per_wave"] >= pairs


def test_page_masks_are_read_when_the_batch_is_created():
    w = dict(workloads())["ragged"]
    b = w.batch
    ctx = planner_for(w)
    before = ctx.batch_create(b)
    r = 8  # the single-token request over 700 prior tokens with a sparse mask of its own
    pages = b.page_ids[b.page_indptr[r]:b.page_indptr[r + 1]]
    hidden = {int(p): 0 for p in pages[:20]}          # no token of these pages stays visible
    hidden[int(pages[20])] = 0x00F0                    # four tokens of this one do
    ctx.mask_kvpage(np.fromiter(hidden.keys(), np.int32), np.fromiter(hidden.values(), np.uint32))
    after = ctx.batch_create(b)
    exp_work, _ = expected_work(w, page_mask=hidden)
    assert after.work()["visited_pages"] == exp_work["visited_pages"] < before.work()["visited_pages"]
    assert before.work()["visited_pages"] == expected_work(w)[0]["visited_pages"]  # the earlier batch keeps what it saw


def status_of(fn):
    with pytest.raises(PieError) as e:
        fn()
    return e.value.status


def test_deserialisation_error_codes():
    w = W.c1_tiny()
    b = w.batch
    ctx = planner_for(w, max_adapters=2, max_lora_rank=8)
    ctx.batch_create(b).destroy()

    def edited(field, index, value, **kw):
        a = np.array(getattr(b, field)).copy()
        a[index] = value
        return clone_batch(b, **{field: a}, **kw)
    assert status_of(lambda: ctx.batch_create(edited("page_ids", 3, w.n_kv_pages))) == -2      # page id out of range
    assert status_of(lambda: ctx.batch_create(edited("page_ids", 0, -1))) == -2
    assert status_of(lambda: ctx.batch_create(edited("in_embed_ids", 1, w.n_embeds))) == -2    # embed id out of range
    assert status_of(lambda: ctx.batch_create(edited("out_embed_ids", 1, -2))) == -2
    assert status_of(lambda: ctx.batch_create(edited("positions", 0, -5))) == -2               # negative position
    assert status_of(lambda: ctx.batch_create(edited("kv_len", 0, 0))) == -1                   # shorter than its new tokens
    assert status_of(lambda: ctx.batch_create(edited("kv_len", 0, 10_000))) == -1              # more KV than pages listed
    assert status_of(lambda: ctx.batch_create(edited("tok_indptr", 0, 1))) == -1               # must start at 0
    assert status_of(lambda: ctx.batch_create(clone_batch(b, positions=None))) == -1           # no positions recorded
    assert status_of(lambda: ctx.batch_create(clone_batch(b, adapter_ids=np.full(b.n_requests, 2, np.int32)))) == -2
    # two tokens writing one (page, slot): request 1 gets request 0's pages and length
    pi = np.array(b.page_indptr)
    pages = np.array(b.page_ids).copy()
    n0 = pi[1] - pi[0]
    assert pi[2] - pi[1] >= n0
    pages[pi[1]:pi[1] + n0] = pages[pi[0]:pi[1]]
    kv = np.array(b.kv_len).copy()
    kv[1] = kv[0]
    clash = clone_batch(b, page_ids=pages, kv_len=kv)
    assert status_of(lambda: ctx.batch_create(clash, validate=True)) == -4
    ctx.batch_create(clash, validate=False).destroy()                                          # only checked on request
    # a batch larger than the context was sized for
    tiny = Pie.planner(w.model, w.n_kv_pages, w.n_embeds, max_batch_tokens=int(b.n_tokens) - 1,
                       max_batch_requests=int(b.n_requests))
    assert status_of(lambda: tiny.batch_create(b)) == -3
    few = Pie.planner(w.model, w.n_kv_pages, w.n_embeds, max_batch_tokens=int(b.n_tokens),
                      max_batch_requests=int(b.n_requests) - 1)
    assert status_of(lambda: few.batch_create(b)) == -3
    # a mask with the wrong number of words
    bm = W.c1_tiny(bitmap=True).batch if "bitmap" in W.c1_tiny.__code__.co_varnames else None
    if bm is not None:
        mi = np.array(bm.mask_indptr).copy()
        mi[-1] -= 1
        assert status_of(lambda: ctx.batch_create(clone_batch(bm, mask_indptr=mi))) == -1


def test_planner_context_refuses_device_work():
    w = W.c1_tiny()
    ctx = planner_for(w)
    pb = ctx.batch_create(w.batch)
    assert status_of(lambda: ctx.forward(0, pb)) == -1
    assert status_of(lambda: ctx.forward_all(pb)) == -1
    assert "plans batches" in str(pytest.raises(PieError, lambda: ctx.forward(0, pb)).value)
    ctx._check(ctx.lib.pie_synchronize(ctx.ctx))  # nothing to wait for
    with pytest.raises(PieError):
        Pie.planner(w.model, w.n_kv_pages, w.n_embeds, 8, 8, wave_slots=3)


def test_a_batch_belongs_to_the_context_that_created_it():
    """A batch carries the ranges, the wave count and (on a device context) the device block of its context: another
    context refuses to run or to destroy it, and a planning context's batch cannot be run at all."""
    w = dict(workloads())["decode64"]
    a, b = planner_for(w), planner_for(w)
    pb = a.batch_create(w.batch)
    assert b.lib.pie_batch_destroy(b.ctx, pb.handle) == -1 and b"another context" in b.lib.pie_last_error(b.ctx)
    assert a.lib.pie_forward(a.ctx, 0, pb.handle) == -1       # planning context: nothing can run
    assert a.lib.pie_forward_all(a.ctx, pb.handle) == -1
    assert a.lib.pie_batch_destroy(None, pb.handle) == -1      # no context at all
    pb.destroy()
    a.close()
    b.close()


def test_pages_of_32_tokens_plan_like_two_blocks_of_16():
    """A KvPage of 32 tokens is two consecutive 16-token blocks: the plan of a batch over pages of 32 equals the plan
    of the same requests over pages of 16 whose tables name blocks 2p, 2p + 1; page sizes other than 16 and 32 are
    refused."""
    m32 = W.ModelDesc(hidden=128, n_q_heads=8, n_kv_heads=2, head_dim=128, mlp_dim=256, vocab=0, page_size=32)
    reqs = [W.RequestSpec(1, 70), W.RequestSpec(1, 31, mask=W.causal_bitmap), W.RequestSpec(45, 37),
            W.RequestSpec(1, 67, prefix_group=0, prefix_len=64), W.RequestSpec(1, 90, prefix_group=0, prefix_len=64),
            W.RequestSpec(1, 600, mask=W.sink_window_mask(4, 40))]
    w32 = W.build_workload("p32", m32, reqs, n_kv_pages=64, seed=12, with_head=False)
    b32 = w32.batch
    b16 = copy.copy(b32)
    b16.page_ids = np.stack([b32.page_ids * 2, b32.page_ids * 2 + 1], axis=1).reshape(-1).astype(np.int32)
    b16.page_indptr = (b32.page_indptr * 2).astype(np.int32)
    m16 = copy.copy(m32)
    m16.page_size = 16
    c32 = Pie.planner(m32, 64, w32.n_embeds, int(b32.n_tokens), int(b32.n_requests))
    c16 = Pie.planner(m16, 128, w32.n_embeds, int(b32.n_tokens), int(b32.n_requests))
    p32, p16 = c32.batch_create(b32, validate=True), c16.batch_create(b16, validate=True)
    assert p32.work() == p16.work() and p32.plan_info() == p16.plan_info()
    assert (p32.prefill_work() == p16.prefill_work()).all()
    # a page mask over all 32 slots hides the same tokens as the two 16-bit halves on the blocks
    c32.mask_kvpage([int(b32.page_ids[0])], [0xFFFF0000])
    c16.mask_kvpage([int(b32.page_ids[0]) * 2, int(b32.page_ids[0]) * 2 + 1], [0x0000, 0xFFFF])
    q32, q16 = c32.batch_create(b32), c16.batch_create(b16)
    assert q32.work() == q16.work() and q32.work() != p32.work()
    for pb in (p32, p16, q32, q16):
        pb.destroy()
    c32.close()
    c16.close()
    for bad in (8, 24, 48):
        mb = copy.copy(m32)
        mb.page_size = bad
        with pytest.raises(PieError) as e:
            Pie.planner(mb, 64, 64, 8, 8)
        assert e.value.status == -7


def test_prefill_requests_over_a_shared_prefix_share_an_xcd():
    """Prefill requests whose page tables begin with the same physical pages (a shared prefix): for every kv head
    their query blocks all run on one XCD, next to each other in its list, so the prefix's K/V pages are fetched
    from HBM once and served by that XCD's L2 afterwards; unrelated requests spread as before."""
    m = small_model(128, 16, 8)
    fam = [W.RequestSpec(96, 512 + 16 * i, prefix_group=0, prefix_len=512) for i in range(5)]
    fam2 = [W.RequestSpec(64, 256, prefix_group=1, prefix_len=256) for i in range(3)]
    solo = [W.RequestSpec(128, 300 + 40 * i) for i in range(24)]
    reqs = solo[:10] + fam + solo[10:] + fam2
    pages = sum((r.n_new + r.prior_len + 15) // 16 for r in reqs) + 8
    w = W.build_workload("fam", m, reqs, n_kv_pages=pages, seed=4300, std=0.02, with_head=False)
    ctx = planner_for(w)
    pb = ctx.batch_create(w.batch, validate=True)
    info = pb.plan_info()
    work = pb.prefill_work()[:info["prefill_workgroups"]]
    fam_of = {10 + i: "a" for i in range(5)}
    fam_of.update({len(reqs) - 3 + i: "b" for i in range(3)})
    xcds, load = {}, np.zeros(8)
    for i, (r, qb, hk) in enumerate(work.tolist()):
        if r >= 0:
            xcds.setdefault((fam_of.get(r, r), hk), set()).add(i % 8)
            load[i % 8] += 1
    assert all(len(v) == 1 for v in xcds.values()), {k: v for k, v in xcds.items() if len(v) > 1}
    assert load.max() <= 1.3 * load.mean()
    for x in range(8):  # a family's blocks for one kv head are contiguous in the XCD's list
        seq = [(fam_of.get(int(r), int(r)), int(h)) for r, q, h in work[x::8] if r >= 0]
        changes = sum(1 for a, c in zip(seq, seq[1:]) if a != c)
        assert changes == len(set(seq)) - 1
    pb.destroy()
    ctx.close()
