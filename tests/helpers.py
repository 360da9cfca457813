"""Shared test helpers: seed the oracle's resource pools from a Workload, compare distributions."""
import copy

import numpy as np

from oracle import pie_oracle as O


def oracle_pools(w):
    """Fresh oracle KvPool / EmbedPool holding the workload's prior KV and input Embeds."""
    m = w.model
    kv = O.KvPool(w.n_kv_pages, m.page_size, m.n_kv_heads, m.head_dim)
    if len(w.prior.page_ids):
        kv.write(w.prior.page_ids, w.prior.slots, w.prior.k_bits, w.prior.v_bits)
    emb = O.EmbedPool(w.n_embeds, m.hidden)
    emb.write(w.batch.in_embed_ids, w.embed_bits)
    return kv, emb


def run_oracle(w, **kw):
    kv, emb = oracle_pools(w)
    res = O.forward(w.model, w.weights, kv, emb, w.batch, **kw)
    return res, kv, emb


def clone_batch(b, **changes):
    nb = copy.copy(b)
    for k, v in changes.items():
        setattr(nb, k, v)
    return nb


def check_topk(ids_gpu, probs_gpu, z_oracle, ids_oracle, probs_oracle, logit_tie=1e-3, rel=2e-3):
    """Top-k comparator: id at rank i must equal the oracle's, unless the two logits involved are
    closer than `logit_tie` (then either order is correct).  Probabilities compared relatively."""
    n, k = ids_oracle.shape
    for r in range(n):
        for i in range(k):
            g, o = int(ids_gpu[r, i]), int(ids_oracle[r, i])
            if g != o:
                assert abs(z_oracle[r, g] - z_oracle[r, o]) < logit_tie, (r, i, g, o, z_oracle[r, g], z_oracle[r, o])
            # probability of the id the GPU reported, against the oracle's full softmax
        zz = z_oracle[r] - z_oracle[r].max()
        p_full = np.exp(zz) / np.exp(zz).sum()
        ref = p_full[ids_gpu[r].astype(np.int64)]
        np.testing.assert_allclose(probs_gpu[r], ref, rtol=rel, atol=1e-9)
        assert len(set(ids_gpu[r].tolist())) == k, "duplicate ids in top-k"


def deep_oracle_pools(dw):
    """Per-layer oracle KvPools holding each layer's prior KV, and an empty EmbedPool (inputs come from embed_txt)."""
    m = dw.base.model
    kvs = []
    for pr in dw.priors:
        kv = O.KvPool(dw.base.n_kv_pages, m.page_size, m.n_kv_heads, m.head_dim)
        if len(pr.page_ids):
            kv.write(pr.page_ids, pr.slots, pr.k_bits, pr.v_bits)
        kvs.append(kv)
    return kvs, O.EmbedPool(dw.base.n_embeds, m.hidden)
