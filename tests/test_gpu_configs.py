"""GPU parity at the full sizes of the benchmark configurations 2-5, in the launch configuration bench.py
times.  Configs 2, 4 and 5 are compared element by element (the oracle finishes them in seconds).  Config 3
(8320 tokens): the attention output of EVERY token, the layer output and the MLP-side intermediates of every
row of two whole prefill requests, of every decode row and of a seeded sample plus the first and last row of
the other prefill requests.  Primary comparison: oracle with bf16 intermediates (the paper's activation
precision); the wide-intermediate oracle is checked alongside.

Each configuration runs twice: with the depth-scaled draw of the two residual-writing projections (unit-scale
outputs) and with the literal draw, every linear weight ~N(0, 0.02): there the layer output has a standard
deviation of about 2.7 (8B shape) or 7 (70B shape), so many elements exceed |y| = 8 and the output format's own
rounding step is above the stated limits; the error is checked against, and printed as a multiple of, the
rounding floor of the oracle's own y (see gpu_helpers.assert_y_close)."""
import time

import numpy as np
import pytest

import workloads as W
from oracle import pie_oracle as O
from gpu_helpers import (appended_positions, assert_bf16_close, assert_close, assert_mlp_stages, assert_y_close, dec,
                         gpu_forward, make_ctx)
from helpers import check_topk, run_oracle

pytestmark = pytest.mark.gpu


def compare_config(w, rows=None, what="", attention_all_rows=False, literal=False):
    from paper_2510_24051_amd import TAP_ACT, TAP_ATTN, TAP_RESID
    t0 = time.time()
    ctx = make_ctx(w)
    pb, stored, y_bits = gpu_forward(ctx, w)
    print(f"    [{what}] GPU setup+forward {time.time() - t0:.1f}s; work {pb.work()}", flush=True)
    t0 = time.time()
    res_b, _, _ = run_oracle(w, rows=rows, round_intermediates=True)
    print(f"    [{what}] oracle (bf16 intermediates) {time.time() - t0:.1f}s on {len(res_b.rows)} rows", flush=True)
    sel = res_b.rows
    out_ids = w.batch.out_embed_ids[sel]
    assert (out_ids >= 0).all()
    y_gpu_bits = ctx.embed_read(out_ids)
    y_gpu = dec(y_gpu_bits)
    # literal draw: the residual projections are sqrt(2 n_layers) times the depth-scaled ones
    scale = float(np.sqrt(2.0 * w.model.n_layers)) if literal else 1.0
    assert_y_close(y_gpu, res_b.y, f"{what} y vs oracle (bf16 intermediates)", allow_scale=scale)
    res_a, _, _ = run_oracle(w, rows=rows)
    assert_y_close(y_gpu, res_a.y, f"{what} y vs oracle (wide intermediates)", stored_as=res_b.y, allow_scale=scale)
    m, T = w.model, w.batch.n_tokens
    o_gpu = dec(ctx.read_tap(TAP_ATTN, T)).reshape(T, m.n_q_heads, m.head_dim)
    if attention_all_rows:
        t0 = time.time()
        res_o, _, _ = run_oracle(w, round_intermediates=True, attention_only=True)
        print(f"    [{what}] oracle attention of all {T} rows {time.time() - t0:.1f}s", flush=True)
        assert_close(o_gpu, res_o.o, f"{what} attention output, all {T} rows", 2e-2, 2e-3)
    else:
        assert_close(o_gpu[sel], res_b.o, f"{what} attention output", 2e-2, 2e-3)
    # the fp32 residual after the attention block and the SwiGLU activation (the down projection's input): what
    # the wide gate/up and down kernels produce is checked where it is made, not only through y
    h_gpu = ctx.read_tap(TAP_RESID, T)[sel]
    assert_close(h_gpu, res_b.h, f"{what} residual after attention", 2e-2, 2e-3)
    act_bits = ctx.read_tap(TAP_ACT, T)[sel]
    act_gpu = dec(act_bits)
    assert_mlp_stages(w, h_gpu, act_bits, y_gpu_bits, sel, what)
    assert_close(act_gpu, res_b.act, f"{what} SwiGLU activation", 2e-2 * max(1.0, np.abs(res_b.act).max()),
                 2e-3 * max(1.0, np.abs(res_b.act).mean() * 4))
    pages, slots = appended_positions(w)
    k_gpu, v_gpu = ctx.kv_read(0, pages, slots)
    assert_bf16_close(k_gpu, res_b.k_new, f"{what} appended K", ulps=2)
    assert_bf16_close(v_gpu, res_b.v_new, f"{what} appended V", ulps=2)
    if w.head is not None and len(w.dist_rows):
        ids_e = w.batch.out_embed_ids[w.dist_rows]
        gi, gp = ctx.get_next_dist(ids_e, w.top_k, w.temperature)
        emb = O.EmbedPool(w.n_embeds, m.hidden)
        emb.write(ids_e, ctx.embed_read(ids_e))
        t0 = time.time()
        oi, op, z = O.get_next_dist(m, w.head, emb, ids_e, w.top_k, w.temperature, round_intermediates=True)
        check_topk(gi, gp, z / w.temperature, oi, op)
        print(f"    {what} top-{w.top_k} over {m.vocab}: ids identical {np.mean(gi == oi) * 100:.2f}% "
              f"(rest within the 1e-3 logit tie rule), oracle {time.time() - t0:.1f}s", flush=True)
    ctx.close()


LITERAL = pytest.mark.parametrize("literal", [False, True], ids=["depth_scaled", "literal"])


@LITERAL
def test_c2_decode_full(literal):
    w = W.c2_decode(with_head=False, literal=literal)
    compare_config(w, what="c2 literal" if literal else "c2", literal=literal)


@pytest.mark.parametrize("n_requests", [17, 45])
def test_8b_shape_ragged_row_counts(n_requests):
    """The 8B-shaped layer with row counts that leave the last 32-row block of the weight-streaming GEMMs ragged:
    17 rows (one block, two-wave gate/up workgroups) and 45 rows (two blocks, the eight-wave gate/up workgroups that
    split K inside the workgroup).  Shorter contexts than configuration 2 keep the oracle quick."""
    w = W.c2_decode(seed=2100 + n_requests, n_requests=n_requests, ctx_lo=40, ctx_hi=700, n_kv_pages=4096,
                    with_head=False)
    compare_config(w, what=f"8B shape, {n_requests} rows")


def c3_rows(b, whole_requests, n_sample):
    rng = np.random.default_rng(3)
    n_prefill_tok = int(b.tok_indptr[8])
    sample = np.sort(rng.choice(n_prefill_tok, size=n_sample, replace=False))
    edges = np.concatenate([b.tok_indptr[:8], b.tok_indptr[1:9] - 1])  # first and last token of every prefill
    whole = np.concatenate([np.arange(b.tok_indptr[r], b.tok_indptr[r + 1]) for r in whole_requests])
    return np.unique(np.concatenate([sample, edges, whole, np.arange(n_prefill_tok, b.n_tokens)]))


def test_c3_mixed_all_attention_rows_and_whole_requests():
    w = W.c3_mixed()
    b = w.batch
    prior = b.kv_len[:8] - 1024
    whole = [int(np.argmin(prior)), int(np.argmax(prior))]  # the shortest and the longest prior context
    print(f"    [c3] prefill priors {prior.tolist()}, every row of requests {whole}", flush=True)
    compare_config(w, rows=c3_rows(b, whole, 96), what="c3", attention_all_rows=True)


def test_c3_mixed_literal_sampled():
    w = W.c3_mixed(literal=True, with_head=False)
    compare_config(w, rows=c3_rows(w.batch, [5], 96), what="c3 literal", literal=True)


@LITERAL
def test_c4_prefix_tree_full(literal):
    w = W.c4_prefix_tree(literal=literal)
    compare_config(w, what="c4 literal" if literal else "c4", literal=literal)


@LITERAL
def test_c5_sparse_long_full(literal):
    w = W.c5_sparse_long(literal=literal, with_head=not literal)
    compare_config(w, what="c5 literal" if literal else "c5", literal=literal)
