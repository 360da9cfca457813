"""GPU parity on seeded random small configurations: head grouping, head size, request mixes, masks of every
density, shared prefixes, in-place Embeds and dropped rows drawn at random (all inputs valid), one layer each,
compared element by element like the hand-picked cases."""
import numpy as np
import pytest

import workloads as W
from test_gpu_parity import compare_layer, random_mask

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng(seed)
    D = int(rng.choice([64, 128]))
    G = int(rng.choice([1, 2, 4, 8]))
    n_kv = int(rng.choice([1, 2, 4]))
    hidden = int(rng.choice([128, 192, 256]))
    mlp = int(rng.choice([256, 320, 512]))
    m = W.ModelDesc(hidden=hidden, n_q_heads=G * n_kv, n_kv_heads=n_kv, head_dim=D, mlp_dim=mlp, vocab=512,
                    page_size=16, rms_eps=1e-5, rope_theta=1e4, n_layers=1)
    P = 16
    reqs, pages = [], 0
    n_groups = int(rng.integers(0, 3))
    group_len = [int(rng.integers(1, 6)) * P for _ in range(n_groups)]
    for _ in range(int(rng.integers(3, 14))):
        kind = rng.random()
        n_new = 1 if kind < 0.55 else (int(rng.integers(2, 6)) if kind < 0.7 else int(rng.integers(6, 90)))
        prior = int(rng.integers(0, 400)) if rng.random() < 0.8 else 0
        kw = {}
        if n_groups and rng.random() < 0.5:
            g = int(rng.integers(0, n_groups))
            prior = group_len[g] + (int(rng.integers(0, 60)) if rng.random() < 0.7 else 0)
            kw.update(prefix_group=g, prefix_len=group_len[g])
        mk = rng.random()
        if mk < 0.25:
            kw["mask"] = random_mask(float(rng.choice([0.02, 0.3, 0.9])))
        elif mk < 0.35:
            kw["mask"] = W.causal_bitmap
        if rng.random() < 0.2:
            kw["in_place"] = True
        if rng.random() < 0.2:
            kw["store_all_rows"] = False
        reqs.append(W.RequestSpec(n_new, prior, **kw))
        pages += (prior + n_new + P - 1) // P
    return m, reqs, pages + 8


# 124, 159, 289 and 314 are the draws of a 210-seed sweep that once fell outside the limits: 124 has outputs with
# |y| >= 8 (the format's half-ulp there is 0.031), 289 a 2%-dense bitmap (a handful of visible keys per row: the
# softmax weights' bf16 rounding showed until their normaliser was summed from the rounded weights), 159 and 314
# exceeded the mean limit against the wide-intermediate oracle.
@pytest.mark.parametrize("seed", [11, 12, 13, 14, 15, 16, 17, 18, 19, 20, 124, 159, 289, 314])
def test_random_small_configurations(seed):
    m, reqs, n_pages = draw_case(seed)
    std = 0.05 * np.sqrt(128.0 / m.hidden)  # the same output scale at every width (the tolerance is absolute)
    w = W.build_workload("random", m, reqs, n_kv_pages=n_pages, seed=8000 + seed, std=std)
    desc = f"seed {seed}: D{m.head_dim} {m.n_q_heads}/{m.n_kv_heads} H{m.hidden} I{m.mlp_dim}, " \
           f"{len(reqs)} requests, T={w.batch.n_tokens}"
    print("  " + desc, flush=True)
    compare_layer(w, what=f"random {seed}")
