"""CPU pins for LoRA adapters in the oracle's `forward` (`forward_with_adapter`)."""
import copy

import numpy as np
import torch
import torch.nn.functional as F

import workloads as W
from oracle import pie_oracle as O
from helpers import clone_batch, deep_oracle_pools, oracle_pools
from test_oracle_forward import dec, small_model, small_workload

ALL = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")


def torch_layer_f64(model, Wt, g1, g2, x, pos):
    """Textbook pre-norm Llama layer for one contiguous causal sequence from float64 weight tensors."""
    H, Hq, Hkv, D = model.hidden, model.n_q_heads, model.n_kv_heads, model.head_dim
    xn = F.rms_norm(x, (H,), g1, eps=model.rms_eps)
    q = F.linear(xn, Wt["wq"]).view(-1, Hq, D)
    k = F.linear(xn, Wt["wk"]).view(-1, Hkv, D)
    v = F.linear(xn, Wt["wv"]).view(-1, Hkv, D)
    freq = model.rope_theta ** (-torch.arange(0, D, 2, dtype=torch.float64) / D)
    ang = pos[:, None] * freq

    def rot(a):
        lo, hi = a[..., : D // 2], a[..., D // 2:]
        c, s = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]
        return torch.cat([lo * c - hi * s, hi * c + lo * s], dim=-1)
    q, k = rot(q), rot(k)
    k = torch.from_numpy(O.bf16_round(k.numpy()))  # KvPages are bf16 storage
    v = torch.from_numpy(O.bf16_round(v.numpy()))
    g = Hq // Hkv
    o = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], k.permute(1, 0, 2).repeat_interleave(g, 0)[None],
                                       v.permute(1, 0, 2).repeat_interleave(g, 0)[None], is_causal=True)
    o = o[0].permute(1, 0, 2).reshape(-1, Hq * D)
    h = x + F.linear(o, Wt["wo"])
    hn = F.rms_norm(h, (H,), g2, eps=model.rms_eps)
    return h + F.linear(F.silu(F.linear(hn, Wt["wgate"])) * F.linear(hn, Wt["wup"]), Wt["wdown"])


def test_adapter_equals_merged_weights():
    m = small_model()
    w = W.build_workload("one", m, [W.RequestSpec(19, 0)], n_kv_pages=8, seed=3, std=0.2)
    ad = W.make_adapter(m, 3, 0, rank=5, projections=ALL, scale=1.7, std=0.2)[0]
    kv, emb = oracle_pools(w)
    res = O.forward(m, w.weights, kv, emb, w.batch, adapters={0: ad}, adapter_ids=[0])
    merged = {}
    for name in ALL:
        base = dec(getattr(w.weights, name))
        a, b, s = ad[name]
        merged[name] = torch.from_numpy(base + s * dec(b) @ dec(a))
    x = torch.from_numpy(dec(w.embed_bits))
    pos = torch.from_numpy(w.batch.positions.astype(np.float64))
    ref = torch_layer_f64(m, merged, torch.from_numpy(dec(w.weights.g1)), torch.from_numpy(dec(w.weights.g2)), x, pos)
    np.testing.assert_allclose(res.y, ref.numpy(), rtol=1e-6, atol=2e-3)
    assert np.mean(np.abs(res.y - ref.numpy())) < 1e-5
    plain = O.forward(m, w.weights, *oracle_pools(w), w.batch)
    assert np.abs(plain.y - res.y).max() > 1e-2  # the adapter matters


def test_zero_update_is_a_no_op():
    w = small_workload()
    m = w.model
    plain = O.forward(m, w.weights, *oracle_pools(w), w.batch)
    ad = W.make_adapter(m, 5, 0, rank=4, projections=ALL, std=0.2)[0]
    zero_b = {k: (a, np.zeros_like(b), s) for k, (a, b, s) in ad.items()}
    zero_s = {k: (a, b, 0.0) for k, (a, b, s) in ad.items()}
    for d in (zero_b, zero_s, {}):
        res = O.forward(m, w.weights, *oracle_pools(w), w.batch, adapters={0: d}, adapter_ids=[0, 0, 0])
        assert np.array_equal(res.y, plain.y)
        assert np.array_equal(res.k_new, plain.k_new)


def test_requests_choose_their_adapter_independently():
    w = small_workload()
    m, b = w.model, w.batch
    ads = {0: W.make_adapter(m, 6, 0, rank=4, projections=ALL, std=0.2)[0],
           3: W.make_adapter(m, 6, 3, rank=7, projections=("wq", "wv", "wdown"), std=0.2)[0]}
    mixed = O.forward(m, w.weights, *oracle_pools(w), b, adapters=ads, adapter_ids=[0, -1, 3])
    plain = O.forward(m, w.weights, *oracle_pools(w), b)
    only0 = O.forward(m, w.weights, *oracle_pools(w), b, adapters=ads, adapter_ids=[0, -1, -1])
    only3 = O.forward(m, w.weights, *oracle_pools(w), b, adapters=ads, adapter_ids=[-1, -1, 3])
    t = b.tok_indptr
    np.testing.assert_allclose(mixed.y[t[0]:t[1]], only0.y[t[0]:t[1]], rtol=1e-12, atol=1e-13)
    assert np.array_equal(mixed.y[t[1]:t[2]], plain.y[t[1]:t[2]])  # the request without adapter is the plain call
    np.testing.assert_allclose(mixed.y[t[2]:t[3]], only3.y[t[2]:t[3]], rtol=1e-12, atol=1e-13)
    assert np.abs(mixed.y[t[0]:t[1]] - plain.y[t[0]:t[1]]).max() > 1e-3
    assert np.abs(mixed.y[t[2]:t[3]] - plain.y[t[2]:t[3]]).max() > 1e-3
    # keys and values appended for an adapted request carry the update
    assert not np.array_equal(mixed.k_new[t[0]:t[1]], plain.k_new[t[0]:t[1]])
    assert np.array_equal(mixed.k_new[t[1]:t[2]], plain.k_new[t[1]:t[2]])
    assert np.array_equal(mixed.k_new[t[2]:t[3]], plain.k_new[t[2]:t[3]])  # adapter 3 has no pair for k


def test_adapters_through_all_layers():
    m = small_model(n_layers=3)
    dw = W.build_deep_workload("deep_ad", m, [W.RequestSpec(1, 21), W.RequestSpec(9, 0)], n_kv_pages=16, seed=21, std=0.2)
    b = dw.base.batch
    ad = W.make_adapter(m, 21, 1, rank=6, projections=ALL, std=0.2)
    kvs, emb = deep_oracle_pools(dw)
    O.embed_txt(dw.table_bits, dw.token_ids, b.positions, emb, b.in_embed_ids)
    res = O.forward_model(m, dw.layers, kvs, emb, b, adapters={1: ad}, adapter_ids=[1, -1])
    # the same by hand: layer by layer with that layer's pairs
    kvs2, emb2 = deep_oracle_pools(dw)
    O.embed_txt(dw.table_bits, dw.token_ids, b.positions, emb2, b.in_embed_ids)
    x = None
    for l in range(3):
        r = O.forward(m, dw.layers[l], kvs2[l], emb2, b, x_in=x, write_embeds=(l == 2), adapters={1: ad[l]}, adapter_ids=[1, -1])
        assert np.array_equal(r.y, res[l].y)
        x = r.y
