"""Seeded synthetic inputs for the batched `forward` / `get_next_dist` hot path.

Pure data: containers and random draws only.  Nothing here computes any step of the layer;
the CPU oracle and the HIP path are both fed from these host arrays and neither is imported.
bf16 tensors are carried as uint16 bit patterns (the draw is made in float32 and rounded once
with torch's CPU cast, a library routine).

The five named workloads follow the shapes of the benchmark configurations (tiny layer; 8B-shaped
decode; 8B-shaped mixed prefill+decode; shared-prefix tree; 70B-shaped sink+window decode).  The
paper's own workloads (Llama-3 text completion, agents, attention-sink inferlets on trained
weights and private prompts) are not available; these random-init tensors stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional

import numpy as np
import torch

# ------------------------------------------------------------------------------------------
# containers
# ------------------------------------------------------------------------------------------


@dataclass
class ModelDesc:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    mlp_dim: int
    vocab: int
    page_size: int = 16
    rms_eps: float = 1e-5
    rope_theta: float = 1e4
    n_layers: int = 1


@dataclass
class LayerWeights:  # uint16 bf16 bits, Linear layout [out, in]; gains [hidden]
    g1: np.ndarray
    wq: np.ndarray
    wk: np.ndarray
    wv: np.ndarray
    wo: np.ndarray
    g2: np.ndarray
    wgate: np.ndarray
    wup: np.ndarray
    wdown: np.ndarray


@dataclass
class HeadWeights:
    g_final: Optional[np.ndarray]  # [hidden] or None (no final norm)
    w_lm: np.ndarray               # [vocab, hidden]


@dataclass
class Batch:  # mirrors the C-ABI batch descriptor, host arrays
    n_requests: int
    n_tokens: int
    tok_indptr: np.ndarray     # int32 [R+1]
    in_embed_ids: np.ndarray   # int32 [T]
    out_embed_ids: np.ndarray  # int32 [T], -1 = row not stored
    positions: np.ndarray      # int32 [T]
    page_indptr: np.ndarray    # int32 [R+1]
    page_ids: np.ndarray       # int32 [sum pages]
    kv_len: np.ndarray         # int32 [R], length after append
    mask_indptr: Optional[np.ndarray] = None  # int64 [R+1] word offsets, None = all inferred causal
    mask_words: Optional[np.ndarray] = None   # uint32
    adapter_ids: Optional[np.ndarray] = None  # int32 [R] LoRA adapter per request, -1 = none


@dataclass
class PriorKV:  # KV tokens present in the pool before the call
    page_ids: np.ndarray  # int32 [n]
    slots: np.ndarray     # int32 [n]
    k_bits: np.ndarray    # uint16 [n, Hkv, D]
    v_bits: np.ndarray    # uint16 [n, Hkv, D]


@dataclass
class RequestSpec:
    n_new: int
    prior_len: int
    mask: Optional[Callable] = None   # (n_new, L, rng) -> bool[n_new, L]; None = inferred causal
    prefix_group: int = -1            # requests with the same group >= 0 alias their first pages
    prefix_len: int = 0               # aliased prefix length in tokens (multiple of page size)
    store_all_rows: bool = True       # False: only the last new token names an output Embed
    in_place: bool = False            # output Embed id == input Embed id


@dataclass
class DeepWorkload:  # the same batch through every layer of a model, inputs produced by embed_txt
    base: "Workload"                  # batch, head, layer-0 weights and prior KV; embed_bits == table[token_ids]
    layers: List[LayerWeights]        # one per layer (layers[0] is base.weights)
    priors: List[PriorKV]             # per-layer prior KV: same (page, slot) list, values of their own
    table_bits: np.ndarray            # uint16 [vocab, H] embedding table
    token_ids: np.ndarray             # int32 [T] input tokens


@dataclass
class Workload:
    name: str
    model: ModelDesc
    n_kv_pages: int
    n_embeds: int
    weights: LayerWeights
    head: Optional[HeadWeights]
    embed_bits: np.ndarray            # uint16 [T, H], row t goes to Embed in_embed_ids[t]
    prior: PriorKV
    batch: Batch
    dist_rows: np.ndarray             # token indices whose output Embed feeds get_next_dist
    top_k: int = 0
    temperature: float = 1.0
    notes: dict = field(default_factory=dict)


# ------------------------------------------------------------------------------------------
# draws
# ------------------------------------------------------------------------------------------

STREAM_WEIGHTS, STREAM_EMBEDS, STREAM_KV, STREAM_PAGES, STREAM_CTX, STREAM_MASK, STREAM_HEAD = 1, 2, 3, 4, 5, 6, 7
STREAM_TABLE, STREAM_TOKENS, STREAM_ADAPTER = 8, 9, 10
LAYER_STREAM_STEP = 100  # layer l > 0 draws its weights / prior KV from stream + l * LAYER_STREAM_STEP


def rng_for(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def normal_bf16(rng: np.random.Generator, shape, std: float = 1.0, mean: float = 0.0,
                chunk: int = 1 << 25) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        x = rng.standard_normal(b - a, dtype=np.float32)
        if std != 1.0:
            x *= np.float32(std)
        if mean != 0.0:
            x += np.float32(mean)
        out[a:b] = to_bf16_bits(x)
    return out.reshape(shape)


def pack_mask_rows(allowed: np.ndarray) -> np.ndarray:
    """bool [n, L] -> uint32 words, row-major, ceil(L/32) words per row, bit j%32 of word j//32."""
    n, L = allowed.shape
    wpr = (L + 31) // 32
    padded = np.zeros((n, wpr * 32), dtype=np.uint8)
    padded[:, :L] = allowed
    by = np.packbits(padded, axis=1, bitorder="little")  # [n, wpr*4] bytes, LSB first
    return by.reshape(n, wpr, 4).copy().view(np.uint32).reshape(-1)


def make_layer_weights(model: ModelDesc, seed: int, std: float = 0.02, resid_std: Optional[float] = None,
                       gain_std: float = 0.02, layer: int = 0) -> LayerWeights:
    """Linear weights ~N(0, std); the two residual-writing projections ~N(0, resid_std);
    norm gains 1 + N(0, gain_std)."""
    rng = rng_for(seed, STREAM_WEIGHTS + layer * LAYER_STREAM_STEP)
    H, Hq, Hkv, D, I = model.hidden, model.n_q_heads, model.n_kv_heads, model.head_dim, model.mlp_dim
    rs = std if resid_std is None else resid_std
    return LayerWeights(
        g1=normal_bf16(rng, (H,), gain_std, 1.0),
        wq=normal_bf16(rng, (Hq * D, H), std),
        wk=normal_bf16(rng, (Hkv * D, H), std),
        wv=normal_bf16(rng, (Hkv * D, H), std),
        wo=normal_bf16(rng, (H, Hq * D), rs),
        g2=normal_bf16(rng, (H,), gain_std, 1.0),
        wgate=normal_bf16(rng, (I, H), std),
        wup=normal_bf16(rng, (I, H), std),
        wdown=normal_bf16(rng, (H, I), rs),
    )


PROJ_SHAPES = {  # projection name -> (out, in) as functions of the model
    "wq": lambda m: (m.n_q_heads * m.head_dim, m.hidden), "wk": lambda m: (m.n_kv_heads * m.head_dim, m.hidden),
    "wv": lambda m: (m.n_kv_heads * m.head_dim, m.hidden), "wo": lambda m: (m.hidden, m.n_q_heads * m.head_dim),
    "wgate": lambda m: (m.mlp_dim, m.hidden), "wup": lambda m: (m.mlp_dim, m.hidden),
    "wdown": lambda m: (m.hidden, m.mlp_dim)}


def make_adapter(model: ModelDesc, seed: int, index: int, rank: int, projections=("wq", "wk", "wv", "wo"),
                 scale: float = 2.0, std: float = 0.02, n_layers: Optional[int] = None):
    """A LoRA adapter: per layer a dict projection -> (A bits [rank, in] ~N(0, std), B bits [out, rank]
    ~N(0, std), scale).  (Trained adapters are not available; a zero-initialised B would change nothing.)"""
    layers = []
    for l in range(n_layers or model.n_layers):
        rng = rng_for(seed, STREAM_ADAPTER + 1000 * index + l * LAYER_STREAM_STEP)
        d = {}
        for name in projections:
            out, inn = PROJ_SHAPES[name](model)
            d[name] = (normal_bf16(rng, (rank, inn), std), normal_bf16(rng, (out, rank), std), float(scale))
        layers.append(d)
    return layers


def make_head_weights(model: ModelDesc, seed: int, std: float = 0.02, gain_std: float = 0.02,
                      final_norm: bool = True) -> HeadWeights:
    rng = rng_for(seed, STREAM_HEAD)
    g = normal_bf16(rng, (model.hidden,), gain_std, 1.0) if final_norm else None
    return HeadWeights(g_final=g, w_lm=normal_bf16(rng, (model.vocab, model.hidden), std))


# ------------------------------------------------------------------------------------------
# generic builder
# ------------------------------------------------------------------------------------------


def build_workload(name: str, model: ModelDesc, requests: List[RequestSpec], n_kv_pages: int, seed: int,
                   weights: Optional[LayerWeights] = None, head: Optional[HeadWeights] = None,
                   std: float = 0.02, resid_std: Optional[float] = None, with_head: bool = True,
                   top_k: int = 0, temperature: float = 1.0, dist_rows: str = "last",
                   n_embeds: Optional[int] = None) -> Workload:
    """Lay out requests over a page pool and draw every tensor.

    Positions: new token i of a request gets position prior_len + i (logical index), prior tokens
    are taken as already rotated.  Page ids are drawn without replacement from the pool; requests
    of one prefix group alias the same physical pages for their first prefix_len tokens.
    """
    P = model.page_size
    R = len(requests)
    rng_pages, rng_ctx, rng_mask = rng_for(seed, STREAM_PAGES), rng_for(seed, STREAM_CTX), rng_for(seed, STREAM_MASK)
    free = rng_pages.permutation(n_kv_pages).astype(np.int32)
    cursor = 0

    def take(n):
        nonlocal cursor
        assert cursor + n <= n_kv_pages, "page pool too small for the workload"
        out = free[cursor:cursor + n]
        cursor += n
        return out

    group_pages = {}
    tok_indptr = np.zeros(R + 1, dtype=np.int32)
    page_indptr = np.zeros(R + 1, dtype=np.int32)
    kv_len = np.zeros(R, dtype=np.int32)
    page_lists, positions, prior_pages, prior_slots = [], [], [], []
    mask_chunks, mask_indptr, any_mask = [], np.zeros(R + 1, dtype=np.int64), False
    for r, rq in enumerate(requests):
        L = rq.prior_len + rq.n_new
        n_pages = (L + P - 1) // P
        shared = np.empty(0, dtype=np.int32)
        first_owner = True
        if rq.prefix_group >= 0:
            assert rq.prefix_len % P == 0 and rq.prefix_len <= rq.prior_len
            if rq.prefix_group not in group_pages:
                group_pages[rq.prefix_group] = take(rq.prefix_len // P)
            else:
                first_owner = False
            shared = group_pages[rq.prefix_group]
        pages = np.concatenate([shared, take(n_pages - len(shared))])
        page_lists.append(pages)
        page_indptr[r + 1] = page_indptr[r] + n_pages
        tok_indptr[r + 1] = tok_indptr[r] + rq.n_new
        kv_len[r] = L
        positions.append(rq.prior_len + np.arange(rq.n_new, dtype=np.int32))
        j0 = 0 if first_owner else len(shared) * P  # prior tokens this request has to seed
        j = np.arange(j0, rq.prior_len, dtype=np.int64)
        prior_pages.append(pages[j // P])
        prior_slots.append((j % P).astype(np.int32))
        if rq.mask is not None:
            allowed = np.asarray(rq.mask(rq.n_new, L, rng_mask), dtype=bool)
            assert allowed.shape == (rq.n_new, L)
            w = pack_mask_rows(allowed)
            mask_chunks.append(w)
            mask_indptr[r + 1] = mask_indptr[r] + len(w)
            any_mask = True
        else:
            mask_indptr[r + 1] = mask_indptr[r]
    T = int(tok_indptr[R])
    n_embeds = n_embeds or max(2 * T, 16)
    rng_e = rng_for(seed, STREAM_EMBEDS)
    ids = rng_e.permutation(n_embeds).astype(np.int32)
    in_ids = ids[:T].copy()
    out_ids = ids[T:2 * T].copy()
    for r, rq in enumerate(requests):
        a, b = tok_indptr[r], tok_indptr[r + 1]
        if rq.in_place:
            out_ids[a:b] = in_ids[a:b]
        if not rq.store_all_rows:
            out_ids[a:b - 1] = -1
    embed_bits = normal_bf16(rng_e, (T, model.hidden), 1.0)

    rng_kv = rng_for(seed, STREAM_KV)
    pp = np.concatenate(prior_pages).astype(np.int32) if prior_pages else np.empty(0, np.int32)
    ps = np.concatenate(prior_slots).astype(np.int32) if prior_slots else np.empty(0, np.int32)
    n_prior = len(pp)
    prior = PriorKV(pp, ps,
                    normal_bf16(rng_kv, (n_prior, model.n_kv_heads, model.head_dim), 1.0),
                    normal_bf16(rng_kv, (n_prior, model.n_kv_heads, model.head_dim), 1.0))
    batch = Batch(
        n_requests=R, n_tokens=T, tok_indptr=tok_indptr, in_embed_ids=in_ids, out_embed_ids=out_ids,
        positions=np.concatenate(positions).astype(np.int32), page_indptr=page_indptr,
        page_ids=np.concatenate(page_lists).astype(np.int32), kv_len=kv_len,
        mask_indptr=mask_indptr if any_mask else None,
        mask_words=(np.concatenate(mask_chunks).astype(np.uint32) if any_mask else None))
    if weights is None:
        weights = make_layer_weights(model, seed, std, resid_std)
    if head is None and with_head and model.vocab > 0:
        head = make_head_weights(model, seed, std)
    if dist_rows == "last":
        rows = tok_indptr[1:] - 1
    elif dist_rows == "decode":
        rows = np.array([tok_indptr[r + 1] - 1 for r, rq in enumerate(requests) if rq.n_new == 1], dtype=np.int32)
    else:
        rows = np.empty(0, dtype=np.int32)
    return Workload(name=name, model=model, n_kv_pages=n_kv_pages, n_embeds=n_embeds, weights=weights, head=head,
                    embed_bits=embed_bits, prior=prior, batch=batch, dist_rows=np.asarray(rows, dtype=np.int32),
                    top_k=top_k, temperature=temperature,
                    notes={"pages_used": cursor, "requests": R, "tokens": T})


def build_deep_workload(name: str, model: ModelDesc, requests: List[RequestSpec], n_kv_pages: int, seed: int,
                        std: float = 0.02, resid_std: Optional[float] = None, top_k: int = 0,
                        n_embeds: Optional[int] = None) -> DeepWorkload:
    """`build_workload` for all `model.n_layers` layers: per-layer weights and prior KV values, an embedding
    table ~N(0,1) and random input tokens whose table rows are the input Embeds."""
    base = build_workload(name, model, requests, n_kv_pages, seed, std=std, resid_std=resid_std, top_k=top_k,
                          n_embeds=n_embeds)
    T = base.batch.n_tokens
    table = normal_bf16(rng_for(seed, STREAM_TABLE), (model.vocab, model.hidden), 1.0)
    tokens = rng_for(seed, STREAM_TOKENS).integers(0, model.vocab, size=T).astype(np.int32)
    base.embed_bits = table[tokens].copy()
    layers, priors = [base.weights], [base.prior]
    n_prior = len(base.prior.page_ids)
    for l in range(1, model.n_layers):
        layers.append(make_layer_weights(model, seed, std, resid_std, layer=l))
        rng_kv = rng_for(seed, STREAM_KV + l * LAYER_STREAM_STEP)
        priors.append(PriorKV(base.prior.page_ids, base.prior.slots,
                              normal_bf16(rng_kv, (n_prior, model.n_kv_heads, model.head_dim), 1.0),
                              normal_bf16(rng_kv, (n_prior, model.n_kv_heads, model.head_dim), 1.0)))
    return DeepWorkload(base=base, layers=layers, priors=priors, table_bits=table, token_ids=tokens)


# ------------------------------------------------------------------------------------------
# mask recipes (return bool [n_new, L])
# ------------------------------------------------------------------------------------------


def causal_bitmap(n_new: int, L: int, rng=None) -> np.ndarray:
    j = np.arange(L)[None, :]
    i = (L - n_new + np.arange(n_new))[:, None]
    return j <= i


def tree_branch_mask(span: int, p_masked: float, prefix_len: int):
    """Every key visible; with probability p_masked one contiguous `span` of the prefix is hidden."""
    def f(n_new, L, rng):
        m = np.ones((n_new, L), dtype=bool)
        if rng.random() < p_masked:
            s = int(rng.integers(0, prefix_len - span + 1))
            m[:, s:s + span] = False
        return m
    return f


def sink_window_mask(n_sink: int, window: int):
    """Attention sink (first n_sink keys) plus a sliding window of the last `window` keys incl. self."""
    def f(n_new, L, rng=None):
        j = np.arange(L)[None, :]
        i = (L - n_new + np.arange(n_new))[:, None]
        return (j <= i) & ((j < n_sink) | (j > i - window))
    return f


# ------------------------------------------------------------------------------------------
# the five named workloads (full size by default; `scale` < 1 shrinks lengths/counts for CPU runs)
# ------------------------------------------------------------------------------------------

def model_tiny() -> ModelDesc:
    return ModelDesc(hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, mlp_dim=512, vocab=1024,
                     page_size=16, rms_eps=1e-5, rope_theta=1e4, n_layers=1)


def model_8b(vocab: int = 128256) -> ModelDesc:
    return ModelDesc(hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, mlp_dim=14336, vocab=vocab,
                     page_size=16, rms_eps=1e-5, rope_theta=5e5, n_layers=32)


def model_70b(vocab: int = 128256) -> ModelDesc:
    return ModelDesc(hidden=8192, n_q_heads=64, n_kv_heads=8, head_dim=128, mlp_dim=28672, vocab=vocab,
                     page_size=16, rms_eps=1e-5, rope_theta=5e5, n_layers=80)


def _resid_std(model: ModelDesc, literal: bool = False) -> Optional[float]:
    """Standard deviation of the two residual-writing projections: depth-scaled (0.02 / sqrt(2 n_layers)), which
    keeps the layer output at unit scale, or with `literal` the same N(0, 0.02) as every other weight (the layer
    output then has a standard deviation of about 2.7 at the 8B shape and 7 at the 70B shape)."""
    return None if literal else 0.02 / float(np.sqrt(2.0 * model.n_layers))


def c1_tiny(seed: int = 1000, bitmap: bool = False) -> Workload:
    m = model_tiny()
    mk = causal_bitmap if bitmap else None
    reqs = [RequestSpec(1, c, mask=mk, in_place=True) for c in (17, 40, 64, 100)] + [RequestSpec(32, 0, mask=mk)]
    return build_workload("c1_tiny", m, reqs, n_kv_pages=32, seed=seed, std=0.02, top_k=8, n_embeds=96)


def c2_decode(seed: int = 2000, n_requests: int = 64, ctx_lo: int = 512, ctx_hi: int = 4096,
              n_kv_pages: int = 40000, model: Optional[ModelDesc] = None, with_head: bool = True,
              weights=None, head=None, top_k: int = 256, literal: bool = False) -> Workload:
    m = model or model_8b()
    ctx = rng_for(seed, STREAM_CTX).integers(ctx_lo, ctx_hi + 1, size=n_requests)
    reqs = [RequestSpec(1, int(c), in_place=True) for c in ctx]
    return build_workload("c2_decode", m, reqs, n_kv_pages, seed, resid_std=_resid_std(m, literal), with_head=with_head,
                          weights=weights, head=head, top_k=top_k)


def c3_mixed(seed: int = 3000, n_prefill: int = 8, prefill_len: int = 1024, prior_hi: int = 2048,
             n_decode: int = 128, decode_ctx: int = 2048, n_kv_pages: int = 40000,
             model: Optional[ModelDesc] = None, with_head: bool = True, weights=None, head=None,
             literal: bool = False) -> Workload:
    m = model or model_8b()
    pri = rng_for(seed, STREAM_CTX).integers(0, prior_hi + 1, size=n_prefill)
    reqs = [RequestSpec(prefill_len, int(p)) for p in pri] + \
           [RequestSpec(1, decode_ctx, in_place=True) for _ in range(n_decode)]
    return build_workload("c3_mixed", m, reqs, n_kv_pages, seed, resid_std=_resid_std(m, literal), with_head=with_head,
                          weights=weights, head=head, top_k=32, dist_rows="decode")


def c4_prefix_tree(seed: int = 4000, n_branches: int = 256, prefix_len: int = 4096, suffix_prior: int = 63,
                   span: int = 512, n_kv_pages: int = 2048, model: Optional[ModelDesc] = None,
                   with_head: bool = False, weights=None, head=None, literal: bool = False) -> Workload:
    m = model or model_8b()
    hidden = set(rng_for(seed, STREAM_CTX).permutation(n_branches)[: n_branches // 4].tolist())  # exactly 25%
    reqs = [RequestSpec(1, prefix_len + suffix_prior, prefix_group=0, prefix_len=prefix_len, in_place=True,
                        mask=tree_branch_mask(span, 1.0 if b in hidden else 0.0, prefix_len))
            for b in range(n_branches)]
    return build_workload("c4_prefix_tree", m, reqs, n_kv_pages, seed, resid_std=_resid_std(m, literal), with_head=with_head,
                          weights=weights, head=head, top_k=0, dist_rows="none")


def c5_sparse_long(seed: int = 5000, n_requests: int = 16, ctx: int = 32768, n_sink: int = 4, window: int = 4096,
                   n_kv_pages: int = 40000, model: Optional[ModelDesc] = None, with_head: bool = True,
                   weights=None, head=None, literal: bool = False) -> Workload:
    m = model or model_70b()
    mk = sink_window_mask(n_sink, window)
    reqs = [RequestSpec(1, ctx, mask=mk, in_place=True) for _ in range(n_requests)]
    return build_workload("c5_sparse_long", m, reqs, n_kv_pages, seed, resid_std=_resid_std(m, literal), with_head=with_head,
                          weights=weights, head=head, top_k=50)


def deep_tiny(seed: int = 6000, n_layers: int = 3, bitmap: bool = False) -> DeepWorkload:
    """The tiny model's mixed batch (4 decode requests + one 32-token prefill) through `n_layers` layers."""
    m = model_tiny()
    m.n_layers = n_layers
    mk = causal_bitmap if bitmap else None
    reqs = [RequestSpec(1, c, mask=mk, in_place=True) for c in (17, 40, 64, 100)] + [RequestSpec(32, 0, mask=mk)]
    return build_deep_workload("deep_tiny", m, reqs, n_kv_pages=32, seed=seed, std=0.02, resid_std=_resid_std(m),
                               top_k=8, n_embeds=96)
