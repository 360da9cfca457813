"""CPU pins for the oracle's `embed_txt` handler and for `forward` through every layer of a model."""
import copy

import numpy as np
import torch

import workloads as W
from oracle import pie_oracle as O
from helpers import clone_batch, deep_oracle_pools
from test_oracle_forward import dec, small_model, torch_llama_layer


def small_deep(seed=21, n_layers=3, reqs=None, std=0.2, **kw):
    m = small_model(n_layers=n_layers)
    reqs = reqs or [W.RequestSpec(1, 21), W.RequestSpec(9, 0), W.RequestSpec(5, 30)]
    return W.build_deep_workload("small_deep", m, reqs, n_kv_pages=64, seed=seed, std=std, top_k=5, **kw)


# ---------------------------------------------------------------- embed_txt
def test_embed_txt_is_a_one_hot_product_and_records_positions():
    dw = small_deep()
    b = dw.base.batch
    _, emb = deep_oracle_pools(dw)
    O.embed_txt(dw.table_bits, dw.token_ids, b.positions, emb, b.in_embed_ids)
    V = dw.base.model.vocab
    onehot = np.zeros((b.n_tokens, V))
    onehot[np.arange(b.n_tokens), dw.token_ids] = 1.0
    ref = onehot @ dec(dw.table_bits)  # exact: one term per output
    assert np.array_equal(dec(emb.read(b.in_embed_ids)), ref)
    assert np.array_equal(emb.pos[b.in_embed_ids], b.positions)
    untouched = np.setdiff1d(np.arange(dw.base.n_embeds), b.in_embed_ids)
    assert (emb.bits[untouched] == 0).all() and (emb.pos[untouched] == -1).all()


def test_positions_recorded_by_embed_txt_equal_explicit_positions():
    dw = small_deep()
    b = dw.base.batch
    kvs, emb = deep_oracle_pools(dw)
    O.embed_txt(dw.table_bits, dw.token_ids, b.positions, emb, b.in_embed_ids)
    a = O.forward(dw.base.model, dw.layers[0], copy.deepcopy(kvs[0]), copy.deepcopy(emb), b)
    c = O.forward(dw.base.model, dw.layers[0], copy.deepcopy(kvs[0]), copy.deepcopy(emb), clone_batch(b, positions=None))
    assert np.array_equal(a.y, c.y)
    # different recorded positions change the result (the rotary step really reads them)
    emb2 = copy.deepcopy(emb)
    O.embed_txt(dw.table_bits, dw.token_ids, b.positions + 3, emb2, b.in_embed_ids)
    d = O.forward(dw.base.model, dw.layers[0], copy.deepcopy(kvs[0]), emb2, clone_batch(b, positions=None))
    assert np.abs(d.y - a.y).max() > 1e-6


# ---------------------------------------------------------------- full depth
def run_deep(dw, batch=None, **kw):
    kvs, emb = deep_oracle_pools(dw)
    b = batch or dw.base.batch
    O.embed_txt(dw.table_bits, dw.token_ids, dw.base.batch.positions, emb, dw.base.batch.in_embed_ids)
    res = O.forward_model(dw.base.model, dw.layers, kvs, emb, b, **kw)
    return res, kvs, emb


def test_model_matches_torch_textbook_stack():
    m = small_model(n_layers=4)
    dw = W.build_deep_workload("one", m, [W.RequestSpec(23, 0)], n_kv_pages=8, seed=3, std=0.2)
    res, kvs, emb = run_deep(dw)
    x = torch.from_numpy(dec(dw.table_bits[dw.token_ids]))
    pos = torch.from_numpy(dw.base.batch.positions.astype(np.float64))
    for l, w in enumerate(dw.layers):
        x = torch_llama_layer(m, w, x, pos)
        np.testing.assert_allclose(res[l].y, x.numpy(), rtol=1e-6, atol=4e-3)
        assert np.mean(np.abs(res[l].y - x.numpy())) < 3e-5
    got = dec(emb.read(dw.base.batch.out_embed_ids))
    assert np.array_equal(got, O.bf16_round(res[-1].y))
    # layers differ from each other: a stack that reused one layer's weights or pool would not match
    assert np.abs(res[1].y - res[0].y).max() > 1e-3


def test_one_layer_model_is_the_single_layer_call():
    dw = small_deep(n_layers=1)
    res, _, emb = run_deep(dw)
    kvs, emb2 = deep_oracle_pools(dw)
    emb2.write(dw.base.batch.in_embed_ids, dw.base.embed_bits)
    one = O.forward(dw.base.model, dw.layers[0], kvs[0], emb2, dw.base.batch)
    assert np.array_equal(res[0].y, one.y)
    assert np.array_equal(emb.bits, emb2.bits)


def test_zero_residual_projections_in_every_layer_give_identity():
    dw = small_deep()
    for w in dw.layers:
        w.wo[:] = 0
        w.wdown[:] = 0
    res, _, _ = run_deep(dw)
    assert np.array_equal(res[-1].y, dec(dw.table_bits[dw.token_ids]))


def test_each_layer_appends_to_its_own_pool():
    dw = small_deep()
    res, kvs, _ = run_deep(dw)
    b = dw.base.batch
    P = dw.base.model.page_size
    for l, kv in enumerate(kvs):
        for r in range(b.n_requests):
            t0, t1 = b.tok_indptr[r], b.tok_indptr[r + 1]
            pages = b.page_ids[b.page_indptr[r]:b.page_indptr[r + 1]]
            j = b.kv_len[r] - (t1 - t0) + np.arange(t1 - t0)
            k, v = kv.read(pages[j // P], j % P)
            assert np.array_equal(k, res[l].k_new[t0:t1]) and np.array_equal(v, res[l].v_new[t0:t1])
        # prior tokens of the layer are untouched
        k, v = kv.read(dw.priors[l].page_ids, dw.priors[l].slots)
        assert np.array_equal(k, dw.priors[l].k_bits) and np.array_equal(v, dw.priors[l].v_bits)
    assert not np.array_equal(res[0].k_new, res[1].k_new)


def test_split_prefill_equals_single_call_through_all_layers():
    """Forward API listing: n tokens in one call == n-1 tokens that fill KvPages + 1 token that reads them."""
    m = small_model(n_layers=3)
    n = 9
    dw = W.build_deep_workload("split", m, [W.RequestSpec(n, 0, store_all_rows=False)], n_kv_pages=8, seed=9, std=0.2)
    b = dw.base.batch
    single, _, _ = run_deep(dw)
    kvs, emb = deep_oracle_pools(dw)
    O.embed_txt(dw.table_bits, dw.token_ids, b.positions, emb, b.in_embed_ids)
    none_out = np.full(n - 1, -1, dtype=np.int32)
    first = clone_batch(b, n_tokens=n - 1, tok_indptr=np.array([0, n - 1], np.int32), in_embed_ids=b.in_embed_ids[:n - 1],
                        out_embed_ids=none_out, positions=b.positions[:n - 1], kv_len=np.array([n - 1], np.int32))
    last = clone_batch(b, n_tokens=1, tok_indptr=np.array([0, 1], np.int32), in_embed_ids=b.in_embed_ids[n - 1:],
                       out_embed_ids=b.out_embed_ids[n - 1:], positions=b.positions[n - 1:], kv_len=np.array([n], np.int32))
    O.forward_model(m, dw.layers, kvs, emb, first)
    two = O.forward_model(m, dw.layers, kvs, emb, last)
    np.testing.assert_allclose(two[-1].y[0], single[-1].y[n - 1], rtol=1e-9, atol=1e-11)
