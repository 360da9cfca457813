"""CPU oracle for the batched `forward` handler (one Llama-class decoder layer over a
heterogeneous batch of commands against KvPage page tables with per-token masks and KV append,
and the same call through every layer of the model), for the `embed_txt` handler (token ids and
positions into Embeds), for the KvPage control calls `mask_kvpage` / `copy_kvpage` (token-level
masking and copying of the KV cache) and for the `get_next_dist` handler (vocab softmax truncated
to top-K).

THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, dense NumPy implementation written from the
paper's statement of the two calls (Programming Model and API: Resources; Forward API; Sample
API; Table 1 rows `forward` and `get_next_dist`) plus the textbook Llama decoder layer the paper
names as the supported model family (Implementation).  It shares no code with the HIP path and
must never be imported by the product package.  Only tests, the smoke check and the bench's
`cpu_baseline` leg call it.

Arithmetic: every floating-point step runs in float64 on values that were first rounded to their
bfloat16 storage format (Embeds, KvPages and weights are bf16 resources - Evaluation, Setup).
`round_intermediates=True` additionally rounds, to bf16, the tensors a bf16 matrix-core
pipeline has to materialise between contractions (normalised activations, q/k/v before and
after the rotary step, attention output, SwiGLU activation); the residual stream stays wide.

Parity pins (tests/test_oracle_*.py, all CPU):
  attention core      brute-force per-element loops on tiny shapes; torch CPU
                      scaled_dot_product_attention; hand-derived fixture in tests/golden/
  mask path           explicit lower-triangular bitmap == inferred causal
  page table          page-id permutation, page size 1 vs 16, masked page == omitted page,
                      aliased pages == private copies
  append / split      one call over n tokens == n-1 tokens writing pages + 1 token reading them
  batching            batch composition and order invariance
  rotary step         norm preservation, position 0 identity, D=2 closed form, shift invariance
  norm / SiLU / GEMM  closed forms, torch CPU rms_norm / silu, zero Wo and Wdown -> y == x
  whole layer         torch CPU expression of a textbook Llama layer on one contiguous request
  softmax / top-k     torch.softmax + torch.topk, k=V sums to 1, shift invariance
  embed_txt           one-hot matrix product, positions recorded with the Embed
  adapters            a torch CPU layer with the merged weights W + scale * B A; zero B or scale is a
                      no-op; a request without adapter equals the plain call; two adapters in one
                      batch equal each request run alone
  mask_kvpage         equals the same call with the masked tokens cleared in an explicit bitmap;
                      all-ones mask is a no-op; a fully masked page equals an omitted page
  copy_kvpage         a request over token-wise copied pages equals the request over the originals;
                      bit-exact against a hand-written slot loop, in every layer's pool
  full depth          torch CPU expression of a textbook L-layer Llama on one contiguous request;
                      zero Wo and Wdown in every layer -> output == input; prefill of n tokens ==
                      n-1 tokens writing pages + 1 token reading them, through all layers
Parity unpinned (convention-internal, the paper is silent): rotate-half pairing, K stored after
the rotary step, final norm inside get_next_dist, tie order of equal probabilities.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

# --------------------------------------------------------------------------------------------
# bfloat16 storage format (sign, 8 exponent bits, 7 mantissa bits) as uint16 bit patterns
# --------------------------------------------------------------------------------------------


def bf16_decode(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float64 (exact)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float64 to the nearest bf16-representable value (ties to even), returned as float64.

    Works on the 8-bit significand directly (frexp/rint/ldexp), so there is no double rounding
    through float32.  Inputs here stay far from bf16's overflow/subnormal range; that is asserted.
    """
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)  # x = m * 2**e, 0.5 <= |m| < 1
    y = np.ldexp(np.rint(m * 256.0) / 256.0, e)  # rint: round half to even
    a = np.abs(np.atleast_1d(y))
    a = a[np.isfinite(a) & (a != 0)]
    if np.size(a):
        assert np.all(a < 3.0e38) and np.all(a > 1.2e-38), "value outside bf16 normal range"
    return y


def bf16_encode(x: np.ndarray) -> np.ndarray:
    """float64 -> uint16 bf16 bit patterns (round to nearest even)."""
    y = bf16_round(x).astype(np.float32)  # exact: 8-bit significand fits float32
    return (y.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------------------------------
# resources owned by the inference layer (Resources paragraph; Inference layer)
# --------------------------------------------------------------------------------------------


class EmbedPool:
    """Per-token Embed slots, bf16 storage, `[n_embeds, hidden]`."""

    def __init__(self, n_embeds: int, hidden: int):
        self.bits = np.zeros((n_embeds, hidden), dtype=np.uint16)
        self.pos = np.full(n_embeds, -1, dtype=np.int64)  # sequence position recorded by embed_txt, -1 = none

    def write(self, ids, bits):
        self.bits[np.asarray(ids, dtype=np.int64)] = np.asarray(bits, dtype=np.uint16)

    def read(self, ids) -> np.ndarray:
        return self.bits[np.asarray(ids, dtype=np.int64)].copy()


class KvPool:
    """KvPages: `n_pages` chunks of `page_size` tokens, K and V per kv head, bf16 storage."""

    def __init__(self, n_pages: int, page_size: int, n_kv_heads: int, head_dim: int):
        self.page_size = page_size
        self.k_bits = np.zeros((n_pages, page_size, n_kv_heads, head_dim), dtype=np.uint16)
        self.v_bits = np.zeros((n_pages, page_size, n_kv_heads, head_dim), dtype=np.uint16)
        self.visible = np.ones((n_pages, page_size), dtype=bool)  # token-level page masks set by mask_kvpage

    def write(self, page_ids, slots, k_bits, v_bits):
        p = np.asarray(page_ids, dtype=np.int64)
        s = np.asarray(slots, dtype=np.int64)
        self.k_bits[p, s] = np.asarray(k_bits, dtype=np.uint16)
        self.v_bits[p, s] = np.asarray(v_bits, dtype=np.uint16)

    def read(self, page_ids, slots):
        p = np.asarray(page_ids, dtype=np.int64)
        s = np.asarray(slots, dtype=np.int64)
        return self.k_bits[p, s].copy(), self.v_bits[p, s].copy()


# --------------------------------------------------------------------------------------------
# layer pieces (textbook Llama decoder layer; the paper only names the family)
# --------------------------------------------------------------------------------------------


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x * (mean(x^2) + eps)^(-1/2) * gain, row-wise over the last axis."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x * (1.0 / np.sqrt(ms + eps)) * np.asarray(gain, dtype=np.float64)


def silu(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.float64)
    return z / (1.0 + np.exp(-z))


def rope(a: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rotary position step on `a[n, heads, D]` with explicit integer positions `[n]`.

    Element i (i < D/2) is paired with element i + D/2; the pair is rotated by the angle
    pos * theta**(-2i/D).  Positions are whatever the caller supplies (Forward API: explicit
    sequence positions); they are not derived from where a token is stored.
    """
    a = np.asarray(a, dtype=np.float64)
    n, _, d = a.shape
    half = d // 2
    inv_freq = np.asarray(theta, dtype=np.float64) ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.asarray(positions, dtype=np.float64).reshape(n, 1) * inv_freq.reshape(1, half)
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    lo, hi = a[..., :half], a[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def mask_row_bits(words: np.ndarray, length: int) -> np.ndarray:
    """Unpack one bitmap row (uint32 words, bit j%32 of word j//32, LSB first) to bool[length]."""
    w = np.ascontiguousarray(words, dtype=np.uint32)
    j = np.arange(length, dtype=np.int64)
    return ((w[j >> 5] >> (j & 31).astype(np.uint32)) & np.uint32(1)).astype(bool)


def masked_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, allowed: np.ndarray) -> np.ndarray:
    """softmax over allowed keys of (q.k)/sqrt(D), times v.

    q [n, Hq, D], k/v [L, Hkv, D] (grouped-query: q head h reads kv head h // (Hq/Hkv)),
    allowed bool [n, L].  A row with no allowed key yields zeros.  Returns [n, Hq, D].
    """
    n, hq, d = q.shape
    hkv = k.shape[1]
    g = hq // hkv
    out = np.zeros((n, hq, d), dtype=np.float64)
    scale = 1.0 / math.sqrt(d)
    any_allowed = allowed.any(axis=1)
    for h in range(hq):
        kh = k[:, h // g, :]
        vh = v[:, h // g, :]
        s = (q[:, h, :] @ kh.T) * scale  # [n, L]
        s = np.where(allowed, s, -np.inf)
        m = np.max(s, axis=1, keepdims=True)
        m = np.where(np.isfinite(m), m, 0.0)
        p = np.exp(s - m)  # exp(-inf) = 0 for masked keys
        denom = np.sum(p, axis=1, keepdims=True)
        denom = np.where(denom > 0, denom, 1.0)
        o = (p / denom) @ vh
        out[:, h, :] = np.where(any_allowed[:, None], o, 0.0)
    return out


# --------------------------------------------------------------------------------------------
# forward handler
# --------------------------------------------------------------------------------------------


@dataclass
class ForwardResult:
    rows: np.ndarray      # token indices for which the per-token outputs below were computed
    y: np.ndarray         # [len(rows), H] float64 layer output before bf16 storage
    q: np.ndarray         # [len(rows), Hq, D] query after the rotary step
    o: np.ndarray         # [len(rows), Hq, D] attention output
    h: np.ndarray         # [len(rows), H] residual stream after the attention block
    k_new: np.ndarray     # [T, Hkv, D] uint16: appended K (after the rotary step), bf16 bits
    v_new: np.ndarray     # [T, Hkv, D] uint16: appended V, bf16 bits
    act: Optional[np.ndarray] = None  # [len(rows), I] SwiGLU product silu(gate) * up, the down projection's input


def _maybe_round(x: np.ndarray, on: bool) -> np.ndarray:
    return bf16_round(x) if on else x


PROJECTIONS = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")


def _lora_delta(adapter, name: str, x: np.ndarray) -> np.ndarray:
    """Low-rank update of one projection for the rows x [n, in]: scale * (x A^T) B^T, or 0 when the adapter
    has no pair for this projection.  `adapter` maps projection names to (A bits [r, in], B bits [out, r],
    scale)."""
    if adapter is None or name not in adapter:
        return 0.0
    a_bits, b_bits, scale = adapter[name]
    return float(scale) * ((x @ bf16_decode(a_bits).T) @ bf16_decode(b_bits).T)


def forward(model, weights, kv: KvPool, emb: EmbedPool, batch, *, rows: Optional[Sequence[int]] = None,
            round_intermediates: bool = False, write_embeds: bool = True,
            x_in: Optional[np.ndarray] = None, adapters=None, adapter_ids=None,
            attention_only: bool = False) -> ForwardResult:
    """One decoder layer over a batch of `forward` commands (Forward API; Table 1 `forward`).

    `model`   : hidden, n_q_heads, n_kv_heads, head_dim, mlp_dim, page_size, rms_eps, rope_theta
    `weights` : g1, wq, wk, wv, wo, g2, wgate, wup, wdown - uint16 bf16 bits, Linear layout [out, in]
    `batch`   : n_requests, n_tokens, tok_indptr[R+1], in_embed_ids[T], out_embed_ids[T] (-1: not
                stored), positions[T], page_indptr[R+1], page_ids (input pages then output pages,
                logical order), kv_len[R] (length after append), mask_indptr[R+1] or None (uint32
                word offsets; empty range = infer causal), mask_words.
    `rows`    : restrict the per-token outputs to these token indices (the K/V append is always done
                for every token, since any later token may attend to it).
    `x_in`    : float64 [T, H] layer input that replaces the Embed read (used by `forward_model` for
                the layers after the first, whose input is the previous layer's output).
    `batch.positions` may be None: the positions are then those recorded with the input Embeds by
    `embed_txt` (Forward API: the call works on the sequence positions associated with its resources).
    `attention_only`: stop after the attention step (y, h and act of the result are None, no Embed is written);
                for tests that compare the attention output of many rows without paying for their MLP.
    `adapters`, `adapter_ids`: `forward_with_adapter` (Forward API): request r uses the LoRA adapter
                `adapters[adapter_ids[r]]` (a dict projection name -> (A bits [rank, in], B bits [out, rank],
                scale); -1 = none): every projection that has a pair computes W x + scale * B (A x).  With
                `round_intermediates` q, k and v are rounded to bf16 once as projected and once more after the
                update is added; the update itself and the gate/up sums stay wide.

    Order of effects inside one call: every input Embed is read first; every K/V append lands
    before any attention read; output Embeds are written last.  New token i of a request sits
    at logical KV index kv_len - n_new + i and is stored in page page_ids[index // P], slot
    index % P, independent of its rotary position.
    """
    H, Hq, Hkv, D = model.hidden, model.n_q_heads, model.n_kv_heads, model.head_dim
    P = model.page_size
    T, R = int(batch.n_tokens), int(batch.n_requests)
    tok_indptr = np.asarray(batch.tok_indptr, dtype=np.int64)
    page_indptr = np.asarray(batch.page_indptr, dtype=np.int64)
    page_ids = np.asarray(batch.page_ids, dtype=np.int64)
    kv_len = np.asarray(batch.kv_len, dtype=np.int64)
    if batch.positions is None:
        positions = emb.pos[np.asarray(batch.in_embed_ids, dtype=np.int64)]
        assert (positions >= 0).all(), "an input Embed carries no position"
    else:
        positions = np.asarray(batch.positions, dtype=np.int64)
    assert tok_indptr[0] == 0 and tok_indptr[R] == T

    rnd = round_intermediates
    Wq, Wk, Wv = bf16_decode(weights.wq), bf16_decode(weights.wk), bf16_decode(weights.wv)
    g1, g2 = bf16_decode(weights.g1), bf16_decode(weights.g2)

    # 1-3: read input Embeds, first norm, K/V projections for every token
    if x_in is None:
        x_all = bf16_decode(emb.bits[np.asarray(batch.in_embed_ids, dtype=np.int64)])  # [T, H]
    else:
        x_all = np.asarray(x_in, dtype=np.float64)
        assert x_all.shape == (T, H)
    xn_all = _maybe_round(rmsnorm(x_all, g1, model.rms_eps), rnd)
    k_all = _maybe_round(xn_all @ Wk.T, rnd)
    v_all = _maybe_round(xn_all @ Wv.T, rnd)

    def adapter_of(r):
        if adapters is None or adapter_ids is None or int(adapter_ids[r]) < 0:
            return None
        return adapters[int(adapter_ids[r])]
    for r in range(R):
        ad = adapter_of(r)
        if ad is not None:
            t0, t1 = tok_indptr[r], tok_indptr[r + 1]
            k_all[t0:t1] = _maybe_round(k_all[t0:t1] + _lora_delta(ad, "wk", xn_all[t0:t1]), rnd)
            v_all[t0:t1] = _maybe_round(v_all[t0:t1] + _lora_delta(ad, "wv", xn_all[t0:t1]), rnd)
    k_all = k_all.reshape(T, Hkv, D)
    v_all = v_all.reshape(T, Hkv, D)
    # 4: rotary step on K with the caller's positions
    k_all = rope(k_all, positions, model.rope_theta)
    # 5: append (bf16 storage) - all appends of the batch precede every attention read
    k_new = bf16_encode(k_all)
    v_new = bf16_encode(v_all)
    for r in range(R):
        t0, t1 = tok_indptr[r], tok_indptr[r + 1]
        n_new = t1 - t0
        pages_r = page_ids[page_indptr[r]:page_indptr[r + 1]]
        j = kv_len[r] - n_new + np.arange(n_new, dtype=np.int64)
        assert n_new == 0 or (j[0] >= 0 and (kv_len[r] + P - 1) // P <= len(pages_r))
        kv.write(pages_r[j // P], j % P, k_new[t0:t1], v_new[t0:t1])

    if rows is None:
        rows = np.arange(T, dtype=np.int64)
    rows = np.asarray(rows, dtype=np.int64)
    req_of = np.searchsorted(tok_indptr, rows, side="right") - 1

    q_out = np.zeros((len(rows), Hq, D))
    o_out = np.zeros((len(rows), Hq, D))
    for r in np.unique(req_of):
        sel = np.nonzero(req_of == r)[0]
        t = rows[sel]
        t0, t1 = tok_indptr[r], tok_indptr[r + 1]
        n_new, L = t1 - t0, int(kv_len[r])
        i_new = t - t0
        # 3-4 for the queries of the selected tokens
        q = _maybe_round(xn_all[t] @ Wq.T, rnd)
        if adapter_of(r) is not None:
            q = _maybe_round(q + _lora_delta(adapter_of(r), "wq", xn_all[t]), rnd)
        q = q.reshape(len(t), Hq, D)
        q = _maybe_round(rope(q, positions[t], model.rope_theta), rnd)
        # 6: gather logical KV [0, L) through the page table, build the allowed matrix
        pages_r = page_ids[page_indptr[r]:page_indptr[r + 1]]
        j = np.arange(L, dtype=np.int64)
        kk = bf16_decode(kv.k_bits[pages_r[j // P], j % P])  # [L, Hkv, D]
        vv = bf16_decode(kv.v_bits[pages_r[j // P], j % P])
        allowed = np.zeros((len(t), L), dtype=bool)
        has_bitmap = batch.mask_indptr is not None and batch.mask_indptr[r + 1] > batch.mask_indptr[r]
        if has_bitmap:
            wpr = (L + 31) // 32
            base = int(batch.mask_indptr[r])
            assert int(batch.mask_indptr[r + 1]) - base == wpr * n_new
            for a, i in enumerate(i_new):
                allowed[a] = mask_row_bits(batch.mask_words[base + i * wpr: base + (i + 1) * wpr], L)
        else:  # causal on logical order
            allowed = j[None, :] <= (L - n_new + i_new)[:, None]
        # tokens hidden by mask_kvpage are invisible to every row, whatever the call's own mask says
        allowed = allowed & kv.visible[pages_r[j // P], j % P][None, :]
        o = masked_attention(q, kk, vv, allowed)
        q_out[sel] = q
        o_out[sel] = _maybe_round(o, rnd)

    if attention_only:
        return ForwardResult(rows=rows, y=None, q=q_out, o=o_out, h=None, k_new=k_new, v_new=v_new, act=None)

    # 7-8: output projection + residual, second norm, SwiGLU MLP + residual
    Wo = bf16_decode(weights.wo)
    o_flat = o_out.reshape(len(rows), Hq * D)
    h = x_all[rows] + o_flat @ Wo.T
    sel_of = {int(r): np.nonzero(req_of == r)[0] for r in np.unique(req_of) if adapter_of(r) is not None}
    for r, sel in sel_of.items():
        h[sel] = h[sel] + _lora_delta(adapter_of(r), "wo", o_flat[sel])
    hn = _maybe_round(rmsnorm(h, g2, model.rms_eps), rnd)
    Wg, Wu, Wd = bf16_decode(weights.wgate), bf16_decode(weights.wup), bf16_decode(weights.wdown)
    gate, up = hn @ Wg.T, hn @ Wu.T
    for r, sel in sel_of.items():
        gate[sel] = gate[sel] + _lora_delta(adapter_of(r), "wgate", hn[sel])
        up[sel] = up[sel] + _lora_delta(adapter_of(r), "wup", hn[sel])
    act = _maybe_round(silu(gate) * up, rnd)
    y = h + act @ Wd.T
    for r, sel in sel_of.items():
        y[sel] = y[sel] + _lora_delta(adapter_of(r), "wdown", act[sel])

    # 9: store output Embeds (bf16) for rows that name one
    if write_embeds:
        out_ids = np.asarray(batch.out_embed_ids, dtype=np.int64)[rows]
        keep = out_ids >= 0
        emb.bits[out_ids[keep]] = bf16_encode(y[keep])
    return ForwardResult(rows=rows, y=y, q=q_out, o=o_out, h=h, k_new=k_new, v_new=v_new, act=act)


# --------------------------------------------------------------------------------------------
# embed_txt handler and the forward pass through every layer
# --------------------------------------------------------------------------------------------


def embed_txt(table_bits: np.ndarray, token_ids, positions, emb: EmbedPool, embed_ids) -> None:
    """Embed API `embed_txt(tok, pos, embs)` (Table 1, InputText): Embed `embed_ids[i]` receives row
    `token_ids[i]` of the embedding table `[vocab, hidden]` (bf16 bits, copied unchanged) and the
    sequence position `positions[i]`, which later `forward` calls use for the rotary step."""
    tok = np.asarray(token_ids, dtype=np.int64)
    ids = np.asarray(embed_ids, dtype=np.int64)
    pos = np.asarray(positions, dtype=np.int64)
    assert tok.shape == ids.shape == pos.shape
    assert (tok >= 0).all() and (tok < table_bits.shape[0]).all()
    emb.bits[ids] = np.asarray(table_bits, dtype=np.uint16)[tok]
    emb.pos[ids] = pos


def forward_model(model, layers, kvs, emb: EmbedPool, batch, *, rows: Optional[Sequence[int]] = None,
                  round_intermediates: bool = False, adapters=None, adapter_ids=None):
    """The `forward` call through the whole model (Forward API: the core Transformer forward pass):
    layer l reads and appends to its own KvPage pool `kvs[l]` with the same page table, its input is
    the output of layer l-1 (kept wide: only Embeds, KvPages and weights are bf16 storage), the
    first layer reads the input Embeds and the last one writes the output Embeds.  `rows` restricts
    the last layer's per-token outputs; every earlier layer is computed for all tokens.
    `adapters[a]` is a list with one projection dict per layer (see `forward`).
    Returns the list of per-layer results."""
    assert len(layers) == len(kvs) and len(layers) >= 1
    results = []
    x = None
    for l, (w, kv) in enumerate(zip(layers, kvs)):
        last = l == len(layers) - 1
        ad_l = None if adapters is None else {a: per_layer[l] for a, per_layer in adapters.items()}
        res = forward(model, w, kv, emb, batch, rows=rows if last else None,
                      round_intermediates=round_intermediates, write_embeds=last, x_in=x,
                      adapters=ad_l, adapter_ids=adapter_ids)
        results.append(res)
        x = res.y
    return results


# --------------------------------------------------------------------------------------------
# KvPage control calls
# --------------------------------------------------------------------------------------------


def mask_kvpage(kvs, page_ids, visible_bits) -> None:
    """`mask_kvpage(tgt, mask)` (Table 1, Forward row): sets the token-level mask of each target KvPage.
    `visible_bits[k]` is an integer whose bit s says whether the token in slot s of page `page_ids[k]`
    stays visible; the mask replaces the page's previous one, belongs to the page in every layer
    (`kvs` is the list of per-layer pools) and is honoured by every later `forward` call on top of that
    call's own mask."""
    P = kvs[0].page_size
    for pg, bits in zip(np.asarray(page_ids, dtype=np.int64), np.asarray(visible_bits, dtype=np.int64)):
        row = np.array([(int(bits) >> s) & 1 for s in range(P)], dtype=bool)
        for kv in kvs:
            kv.visible[pg] = row


def copy_kvpage(kvs, src_pages, src_slots, dst_pages, dst_slots) -> None:
    """`copy_kvpage(src, dst)` (Table 1, Allocate row): token-level copy of KV cache contents.  Token k of
    the call is read from (src_pages[k], src_slots[k]) and written to (dst_pages[k], dst_slots[k]), K and V,
    unchanged bits, in every layer; page masks are not copied.  Source and destination tokens are disjoint."""
    sp, ss = np.asarray(src_pages, dtype=np.int64), np.asarray(src_slots, dtype=np.int64)
    dp, ds = np.asarray(dst_pages, dtype=np.int64), np.asarray(dst_slots, dtype=np.int64)
    assert sp.shape == ss.shape == dp.shape == ds.shape
    src = set(zip(sp.tolist(), ss.tolist()))
    dst = list(zip(dp.tolist(), ds.tolist()))
    assert len(set(dst)) == len(dst) and not (src & set(dst)), "source and destination tokens must be disjoint"
    for kv in kvs:
        k, v = kv.k_bits[sp, ss].copy(), kv.v_bits[sp, ss].copy()
        kv.k_bits[dp, ds] = k
        kv.v_bits[dp, ds] = v


# --------------------------------------------------------------------------------------------
# get_next_dist handler
# --------------------------------------------------------------------------------------------


def logits_from_embeds(model, head, emb: EmbedPool, embed_ids, round_intermediates: bool = False) -> np.ndarray:
    """Final norm (when the head carries a gain) and LM head on stored Embeds -> float64 logits.

    `round_intermediates` rounds the normalised activation to bf16 before the LM head, the
    precision the paper states for activations (Evaluation, Setup: weights, KV cache and
    activations in BF16); the logits themselves stay wide."""
    e = bf16_decode(emb.bits[np.asarray(embed_ids, dtype=np.int64)])
    if head.g_final is not None:
        e = _maybe_round(rmsnorm(e, bf16_decode(head.g_final), model.rms_eps), round_intermediates)
    return e @ bf16_decode(head.w_lm).T


def top_k_dist(logits: np.ndarray, top_k: int, temperature: float = 1.0):
    """softmax(logits / temperature) over the whole vocabulary, truncated to the top_k entries.

    Sorted by descending probability, equal probabilities by ascending token id.  The kept
    probabilities are those of the full distribution (no renormalisation over the survivors).
    Returns (ids int32 [n, k], probs float64 [n, k]).
    """
    z = np.asarray(logits, dtype=np.float64) / float(temperature)
    z = z - np.max(z, axis=-1, keepdims=True)
    p = np.exp(z)
    p = p / np.sum(p, axis=-1, keepdims=True)
    n, vocab = p.shape
    ids = np.empty((n, top_k), dtype=np.int32)
    probs = np.empty((n, top_k), dtype=np.float64)
    for i in range(n):
        order = np.lexsort((np.arange(vocab), -z[i]))[:top_k]  # primary -logit, then id
        ids[i] = order
        probs[i] = p[i, order]
    return ids, probs


def get_next_dist(model, head, emb: EmbedPool, embed_ids, top_k: int, temperature: float = 1.0,
                  round_intermediates: bool = False):
    """Sample API `get_next_dist`: next-token distribution of each Embed, truncated to top-K."""
    z = logits_from_embeds(model, head, emb, embed_ids, round_intermediates)
    ids, probs = top_k_dist(z, top_k, temperature)
    return ids, probs, z
