"""CPU pins for the oracle's building blocks: each is checked against something other than the
oracle itself - a torch CPU library routine, a brute-force loop, a closed form, an invariant or
the hand-derived fixture under tests/golden/."""
import json
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import pie_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(7)


# ---------------------------------------------------------------- bf16 storage format
def test_bf16_round_matches_torch_cast():
    x = np.concatenate([rng.standard_normal(20000) * 3, rng.standard_normal(2000) * 1e-3,
                        rng.standard_normal(2000) * 1e4]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16)
    bits = O.bf16_encode(x.astype(np.float64))
    assert np.array_equal(bits, ref.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(O.bf16_decode(bits), ref.to(torch.float64).numpy())


def test_bf16_ties_to_even_and_no_double_rounding():
    # 1 + 2^-8 is exactly halfway between 1 and 1+2^-7 -> rounds to even (1.0)
    assert O.bf16_round(np.array(1.0 + 2.0 ** -8)) == 1.0
    assert O.bf16_round(np.array(1.0 + 3 * 2.0 ** -8)) == 1.0 + 2.0 ** -6
    # just above the tie by less than a float32 ulp: a detour through float32 would land on the tie
    assert O.bf16_round(np.array(1.0 + 2.0 ** -8 + 2.0 ** -40)) == 1.0 + 2.0 ** -7
    # carry into the next binade
    assert O.bf16_round(np.array(1.998046875 + 0.001)) == 2.0
    assert O.bf16_round(np.array(-0.3)) == -O.bf16_round(np.array(0.3))
    assert O.bf16_round(np.array(0.0)) == 0.0


# ---------------------------------------------------------------- norm / activation
def test_rmsnorm_matches_torch_and_closed_form():
    x = rng.standard_normal((5, 64))
    g = rng.uniform(0.5, 1.5, 64)
    ref = F.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), eps=1e-5).numpy()
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-5), ref, rtol=1e-12, atol=1e-14)
    c = 3.0
    out = O.rmsnorm(np.full((1, 8), c), g[:8], 1e-5)
    np.testing.assert_allclose(out[0], g[:8] * c / math.sqrt(c * c + 1e-5), rtol=1e-14)


def test_silu_matches_torch_and_limits():
    z = rng.standard_normal(1000) * 4
    np.testing.assert_allclose(O.silu(z), F.silu(torch.from_numpy(z)).numpy(), rtol=1e-12, atol=1e-15)
    assert O.silu(np.array(0.0)) == 0.0
    assert abs(O.silu(np.array(40.0)) - 40.0) < 1e-12
    assert abs(O.silu(np.array(-40.0))) < 1e-12


# ---------------------------------------------------------------- rotary step
def test_rope_closed_forms():
    a = rng.standard_normal((6, 3, 8))
    pos = np.array([0, 1, 5, 17, 1000, 32768])
    out = O.rope(a, pos, 1e4)
    # position 0 is the identity
    np.testing.assert_array_equal(out[0], a[0])
    # each (i, i + D/2) pair keeps its norm
    n_in = a[..., :4] ** 2 + a[..., 4:] ** 2
    n_out = out[..., :4] ** 2 + out[..., 4:] ** 2
    np.testing.assert_allclose(n_out, n_in, rtol=1e-12)
    # D = 2: a plain rotation of the plane by pos * 1 radians
    v = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    r = O.rope(v, np.array([2, 3]), 1e4)
    np.testing.assert_allclose(r[0, 0], [math.cos(2), math.sin(2)], atol=1e-15)
    np.testing.assert_allclose(r[1, 0], [-math.sin(3), math.cos(3)], atol=1e-15)


def test_rope_matches_complex_formulation():
    # independent formulation: (a_i + 1j*a_{i+D/2}) * exp(1j * pos * theta^(-2i/D))
    d, theta = 16, 5e5
    a = rng.standard_normal((4, 2, d))
    pos = np.array([3, 77, 4096, 31000])
    z = a[..., : d // 2] + 1j * a[..., d // 2:]
    w = np.exp(1j * pos[:, None, None] * (theta ** (-np.arange(d // 2) * 2.0 / d))[None, None, :])
    zr = z * w
    ref = np.concatenate([zr.real, zr.imag], axis=-1)
    np.testing.assert_allclose(O.rope(a, pos, theta), ref, rtol=1e-10, atol=1e-12)


def test_rope_relative_property():
    # the score q.k after rotation depends only on the position difference
    d = 32
    q, k = rng.standard_normal((1, 1, d)), rng.standard_normal((1, 1, d))
    s1 = np.sum(O.rope(q, [10], 1e4) * O.rope(k, [4], 1e4))
    s2 = np.sum(O.rope(q, [1010], 1e4) * O.rope(k, [1004], 1e4))
    assert abs(s1 - s2) < 1e-10


# ---------------------------------------------------------------- mask unpacking
def test_mask_row_bits_lsb_first():
    words = np.array([0b1011, 0x80000000, 1], dtype=np.uint32)
    bits = O.mask_row_bits(words, 70)
    expect = np.zeros(70, dtype=bool)
    expect[[0, 1, 3, 63, 64]] = True
    assert np.array_equal(bits, expect)


# ---------------------------------------------------------------- attention core
def brute_attention(q, k, v, allowed):
    n, hq, d = q.shape
    hkv = k.shape[1]
    out = np.zeros_like(q)
    for t in range(n):
        for h in range(hq):
            g = h // (hq // hkv)
            js = [j for j in range(k.shape[0]) if allowed[t, j]]
            if not js:
                continue
            s = [sum(q[t, h, e] * k[j, g, e] for e in range(d)) / math.sqrt(d) for j in js]
            mx = max(s)
            w = [math.exp(x - mx) for x in s]
            tot = sum(w)
            for e in range(d):
                out[t, h, e] = sum(w[i] * v[j, g, e] for i, j in enumerate(js)) / tot
    return out


def test_attention_vs_brute_force():
    n, L, hq, hkv, d = 3, 11, 4, 2, 8
    q, k, v = rng.standard_normal((n, hq, d)), rng.standard_normal((L, hkv, d)), rng.standard_normal((L, hkv, d))
    allowed = rng.random((n, L)) < 0.6
    allowed[1] = False  # a row with no allowed key -> zeros
    out = O.masked_attention(q, k, v, allowed)
    np.testing.assert_allclose(out, brute_attention(q, k, v, allowed), rtol=1e-12, atol=1e-14)
    assert np.all(out[1] == 0.0)


def test_attention_vs_torch_sdpa():
    n, L, hq, hkv, d = 7, 50, 8, 2, 16
    q, k, v = rng.standard_normal((n, hq, d)), rng.standard_normal((L, hkv, d)), rng.standard_normal((L, hkv, d))
    allowed = rng.random((n, L)) < 0.5
    allowed[:, 0] = True
    g = hq // hkv
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(g, dim=0)[None]
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(g, dim=0)[None]
    ref = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=torch.from_numpy(allowed)[None, None])
    ref = ref[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(O.masked_attention(q, k, v, allowed), ref, rtol=1e-10, atol=1e-12)


def test_attention_special_cases():
    L, d = 9, 4
    k, v = rng.standard_normal((L, 1, d)), rng.standard_normal((L, 1, d))
    q = rng.standard_normal((2, 1, d))
    one = np.zeros((2, L), dtype=bool)
    one[0, 3] = one[1, 7] = True
    out = O.masked_attention(q, k, v, one)  # single allowed key -> that V row exactly
    np.testing.assert_array_equal(out[0, 0], v[3, 0])
    np.testing.assert_array_equal(out[1, 0], v[7, 0])
    allowed = rng.random((2, L)) < 0.7
    allowed[:, 0] = True
    out = O.masked_attention(np.zeros_like(q), k, v, allowed)  # q = 0 -> mean of allowed V rows
    for t in range(2):
        np.testing.assert_allclose(out[t, 0], v[allowed[t], 0].mean(axis=0), rtol=1e-13)


def test_attention_hand_derived_fixture():
    """tests/golden/attention_hand_case.json: numbers derived by hand from the definition."""
    with open(os.path.join(GOLDEN, "attention_hand_case.json")) as f:
        case = json.load(f)
    q = np.array(case["q"], dtype=np.float64).reshape(1, 1, 2)
    q[0, 0, 0] *= math.log(2.0) * math.sqrt(2.0)  # fixture stores q0 in units of ln2*sqrt(2)
    k = np.array(case["k"], dtype=np.float64).reshape(3, 1, 2)
    v = np.array(case["v"], dtype=np.float64).reshape(3, 1, 2)
    for allowed, expect in zip(case["allowed"], case["expected_o"]):
        out = O.masked_attention(q, k, v, np.array([allowed], dtype=bool))
        np.testing.assert_allclose(out[0, 0], expect, rtol=1e-13, atol=1e-15)


# ---------------------------------------------------------------- distribution
def test_top_k_matches_torch():
    n, vocab, k = 4, 777, 13
    z = rng.standard_normal((n, vocab)) * 2
    for temp in (1.0, 0.7, 2.5):
        ids, probs = O.top_k_dist(z, k, temp)
        p = torch.softmax(torch.from_numpy(z) / temp, dim=-1)
        tv, ti = torch.topk(p, k, dim=-1)
        assert np.array_equal(ids, ti.numpy().astype(np.int32))
        np.testing.assert_allclose(probs, tv.numpy(), rtol=1e-12)


def test_top_k_full_vocab_sums_to_one_sorted_and_shift_invariant():
    z = rng.standard_normal((2, 300))
    ids, probs = O.top_k_dist(z, 300)
    np.testing.assert_allclose(probs.sum(axis=1), 1.0, rtol=1e-13)
    assert np.all(np.diff(probs, axis=1) <= 0)
    assert all(sorted(ids[i].tolist()) == list(range(300)) for i in range(2))
    ids2, probs2 = O.top_k_dist(z + 123.25, 300)
    assert np.array_equal(ids, ids2)
    np.testing.assert_allclose(probs, probs2, rtol=1e-12)
    ids8, probs8 = O.top_k_dist(z, 8)  # truncation keeps the full-softmax values, no renormalisation
    assert np.array_equal(ids8, ids[:, :8]) and np.array_equal(probs8, probs[:, :8])
    assert probs8.sum(axis=1).max() < 1.0


def test_top_k_tie_goes_to_lower_id():
    z = np.zeros((1, 10))
    z[0, [7, 2, 5]] = 1.0
    ids, probs = O.top_k_dist(z, 4)
    assert ids[0].tolist() == [2, 5, 7, 0]
    np.testing.assert_allclose(probs[0, 0], math.e / (3 * math.e + 7), rtol=1e-14)
