"""ctypes binding of libpie_mi355.so.  Every method marshals arguments for the C call of the same
name (pie_<method>) and does nothing else: all computation runs in the HIP kernels.  PyTorch is
used for device memory and the stream only.  There is no CPU fallback: a missing library raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libpie_mi355.so"

PIE_N_STAGES = 13
STAGE_NAMES = ["norm1", "qkv", "rope_append", "attn_decode", "attn_prefill", "attn_merge", "oproj", "norm2",
               "gateup", "down", "head_norm", "lm_head", "topk"]
TAP_Q, TAP_ATTN, TAP_RESID, TAP_ACT, TAP_LOGITS = 0, 1, 2, 3, 4

STATUS = {0: "PIE_OK", -1: "PIE_EINVAL", -2: "PIE_ERANGE", -3: "PIE_EBATCH", -4: "PIE_ECONFLICT", -5: "PIE_ENOMEM",
          -6: "PIE_EHIP", -7: "PIE_EUNSUPPORTED"}


class PieError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS.get(status, status)}: {message}")
        self.status = status


class ModelDescC(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("hidden", "n_q_heads", "n_kv_heads", "head_dim", "mlp_dim", "vocab",
                                          "page_size")] + [("rms_eps", C.c_float), ("rope_theta", C.c_float),
                                                           ("n_layers", C.c_int32)]


class PoolDescC(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_kv_pages", "n_embeds", "max_batch_tokens", "max_batch_requests",
                                          "max_top_k", "max_dist_rows", "max_adapters", "max_lora_rank")]


class ForwardBatchC(C.Structure):
    _fields_ = [("n_requests", C.c_int32), ("n_tokens", C.c_int32), ("tok_indptr", C.c_void_p),
                ("in_embed_ids", C.c_void_p), ("out_embed_ids", C.c_void_p), ("positions", C.c_void_p),
                ("page_indptr", C.c_void_p), ("page_ids", C.c_void_p), ("kv_len", C.c_void_p),
                ("mask_indptr", C.c_void_p), ("mask_words", C.c_void_p), ("adapter_ids", C.c_void_p)]


def lib_path() -> str:
    return os.path.join(HERE, _LIB_NAME)


_lib = None


def load_library():
    """Load the built library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: build it with `python -m paper_2510_24051_amd.build` "
                                "(or __graft_entry__.build()); the HIP path has no fallback")
    lib = C.CDLL(path)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    sigs = {
        "pie_create": [C.POINTER(ModelDescC), C.POINTER(PoolDescC), vp, C.POINTER(vp)],
        "pie_destroy": [vp],
        "pie_load_layer": [vp, i32] + [vp] * 9,
        "pie_load_head": [vp, vp, vp],
        "pie_embed_write": [vp, vp, i32, vp],
        "pie_embed_read": [vp, vp, i32, vp],
        "pie_kv_write": [vp, i32, vp, vp, i32, vp, vp],
        "pie_kv_read": [vp, i32, vp, vp, i32, vp, vp],
        "pie_batch_create": [vp, C.POINTER(ForwardBatchC), i32, C.POINTER(vp)],
        "pie_batch_destroy": [vp, vp],
        "pie_forward": [vp, i32, vp],
        "pie_forward_all": [vp, vp],
        "pie_load_embedding": [vp, vp],
        "pie_load_adapter": [vp, i32, i32, i32, i32, f32, vp, vp],
        "pie_embed_txt": [vp, vp, vp, i32, vp],
        "pie_mask_kvpage": [vp, vp, vp, i32],
        "pie_copy_kvpage": [vp, vp, vp, vp, vp, i32],
        "pie_forward_host": [vp, i32, C.POINTER(ForwardBatchC), i32],
        "pie_get_next_dist": [vp, vp, i32, i32, f32, vp, vp],
        "pie_get_next_dist_static": [vp, vp, i32, i32, f32, vp, vp],
        "pie_forward_dist": [vp, vp, vp, i32, i32, f32, vp, vp],
        "pie_synchronize": [vp],
        "pie_read_tap": [vp, i32, vp, i64],
        "pie_set_stage_timing": [vp, i32],
        "pie_stage_times": [vp, vp],
        "pie_batch_work": [vp, vp],
        "pie_batch_plan_info": [vp, vp],
        "pie_batch_prefill_work": [vp, vp, i32, vp],
        "pie_create_planner": [C.POINTER(ModelDescC), C.POINTER(PoolDescC), i32, C.POINTER(vp)],
    }
    for name, args in sigs.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = i32
    lib.pie_last_error.argtypes = [vp]
    lib.pie_last_error.restype = C.c_char_p
    _lib = lib
    return lib


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class PieBatch:
    def __init__(self, owner: "Pie", handle, keepalive):
        self.owner, self.handle, self._keep = owner, handle, keepalive

    def work(self) -> dict:
        out = np.zeros(6, dtype=np.int64)
        self.owner._check(self.owner.lib.pie_batch_work(self.handle, _ptr(out)))
        return {"kv_bytes": int(out[0]), "kv_bytes_decode": int(out[1]), "attn_flops": int(out[2]),
                "visited_pages": int(out[3]), "kv_bytes_unique": int(out[4]), "kv_bytes_requested": int(out[5])}

    def plan_info(self) -> dict:
        out = np.zeros(8, dtype=np.int64)
        self.owner._check(self.owner.lib.pie_batch_plan_info(self.handle, _ptr(out)))
        return {"decode_waves": int(out[0]), "segments": int(out[1]), "max_pairs_per_wave": int(out[2]),
                "prefill_items": int(out[3]), "decode_requests": int(out[4]), "rows_cap": int(out[5]),
                "prefill_workgroups": int(out[6]), "prefill_workgroups_pair_weights": int(out[7])}

    def prefill_work(self) -> np.ndarray:
        """[n, 3] int32 (request, query block, kv head) per workgroup of the two prefill launches, one after the
        other (sizes in plan_info); request -1 = empty."""
        n = C.c_int32(0)
        self.owner._check(self.owner.lib.pie_batch_prefill_work(self.handle, None, 0, C.byref(n)))
        out = np.zeros((max(n.value, 1), 3), dtype=np.int32)
        self.owner._check(self.owner.lib.pie_batch_prefill_work(self.handle, _ptr(out), n.value, C.byref(n)))
        return out[:n.value]

    def destroy(self):
        if self.handle is not None:
            self.owner.lib.pie_batch_destroy(self.owner.ctx, self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class Pie:
    """One context = one GPU = one stream.  bf16 tensors cross this binding as uint16 numpy arrays (host)
    or torch.bfloat16 CUDA tensors (device)."""

    def __init__(self, model, n_kv_pages: int, n_embeds: int, max_batch_tokens: int, max_batch_requests: int,
                 max_top_k: int = 256, max_dist_rows: int = 0, n_layers: int = 1, device: str = "cuda:0",
                 stream: Optional[torch.cuda.Stream] = None, max_adapters: int = 0, max_lora_rank: int = 0):
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the HIP path cannot run (there is no CPU fallback)")
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.stream = stream if stream is not None else torch.cuda.Stream(device=self.device)
        self.model = model
        md = ModelDescC(model.hidden, model.n_q_heads, model.n_kv_heads, model.head_dim, model.mlp_dim, model.vocab,
                        model.page_size, model.rms_eps, model.rope_theta, n_layers)
        pd = PoolDescC(n_kv_pages, n_embeds, max_batch_tokens, max_batch_requests, max_top_k, max_dist_rows,
                       max_adapters, max_lora_rank)
        h = C.c_void_p()
        st = self.lib.pie_create(C.byref(md), C.byref(pd), C.c_void_p(self.stream.cuda_stream), C.byref(h))
        if st != 0:
            raise PieError(st, self.lib.pie_last_error(None).decode())
        self.ctx = h

    @classmethod
    def planner(cls, model, n_kv_pages: int, n_embeds: int, max_batch_tokens: int, max_batch_requests: int,
                n_layers: int = 1, max_adapters: int = 0, max_lora_rank: int = 0, wave_slots: int = 2048) -> "Pie":
        """A context that only deserialises and plans batches (pie_create_planner): needs no GPU.  batch_create,
        PieBatch.work / plan_info and mask_kvpage work on it; everything else raises PieError."""
        self = cls.__new__(cls)
        self.lib = load_library()
        self.device, self.stream, self.model = None, None, model
        md = ModelDescC(model.hidden, model.n_q_heads, model.n_kv_heads, model.head_dim, model.mlp_dim, model.vocab,
                        model.page_size, model.rms_eps, model.rope_theta, n_layers)
        pd = PoolDescC(n_kv_pages, n_embeds, max_batch_tokens, max_batch_requests, 0, 0, max_adapters, max_lora_rank)
        h = C.c_void_p()
        st = self.lib.pie_create_planner(C.byref(md), C.byref(pd), int(wave_slots), C.byref(h))
        if st != 0:
            raise PieError(st, self.lib.pie_last_error(None).decode())
        self.ctx = h
        return self

    # ---- helpers ----
    def _check(self, st: int):
        if st != 0:
            raise PieError(st, self.lib.pie_last_error(self.ctx).decode())

    def _dev_bf16(self, bits) -> torch.Tensor:
        if isinstance(bits, torch.Tensor):
            assert bits.dtype == torch.bfloat16 and bits.is_cuda and bits.is_contiguous()
            return bits
        a = np.ascontiguousarray(bits, dtype=np.uint16)
        t = torch.from_numpy(a.view(np.int16)).to(self.device, non_blocking=False)
        return t.view(torch.bfloat16)

    def close(self):
        if getattr(self, "ctx", None) is not None:
            self.lib.pie_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- weights ----
    def load_layer(self, layer: int, w):
        names = ("g1", "wq", "wk", "wv", "wo", "g2", "wgate", "wup", "wdown")
        ts = [self._dev_bf16(getattr(w, n)) for n in names]
        torch.cuda.synchronize(self.device)
        self._check(self.lib.pie_load_layer(self.ctx, layer, *[C.c_void_p(t.data_ptr()) for t in ts]))
        del ts

    def load_head(self, head):
        g = None if head.g_final is None else self._dev_bf16(head.g_final)
        w = self._dev_bf16(head.w_lm)
        torch.cuda.synchronize(self.device)
        self._check(self.lib.pie_load_head(self.ctx, None if g is None else C.c_void_p(g.data_ptr()),
                                           C.c_void_p(w.data_ptr())))

    def load_embedding(self, table_bits):
        t = self._dev_bf16(table_bits)
        torch.cuda.synchronize(self.device)
        self._check(self.lib.pie_load_embedding(self.ctx, C.c_void_p(t.data_ptr())))

    PROJECTIONS = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")

    def load_adapter(self, adapter: int, layers):
        """`layers[l]` maps projection names to (A bits [rank, in], B bits [out, rank], scale)."""
        for l, d in enumerate(layers):
            for name, (a_bits, b_bits, scale) in d.items():
                a, b = self._dev_bf16(a_bits), self._dev_bf16(b_bits)
                torch.cuda.synchronize(self.device)
                self._check(self.lib.pie_load_adapter(self.ctx, adapter, l, self.PROJECTIONS.index(name), a.shape[0],
                                                      float(scale), C.c_void_p(a.data_ptr()), C.c_void_p(b.data_ptr())))

    # ---- resources ----
    def embed_txt(self, token_ids, positions, embed_ids):
        tok, pos, ids = _i32(token_ids), _i32(positions), _i32(embed_ids)
        if not (len(tok) == len(pos) == len(ids)):
            raise ValueError("embed_txt: token_ids, positions and embed_ids must have one length")
        self._check(self.lib.pie_embed_txt(self.ctx, _ptr(tok), _ptr(pos), len(tok), _ptr(ids)))

    def embed_write(self, embed_ids, bits):
        ids = _i32(embed_ids)
        t = self._dev_bf16(bits)
        torch.cuda.synchronize(self.device)
        self._check(self.lib.pie_embed_write(self.ctx, _ptr(ids), len(ids), C.c_void_p(t.data_ptr())))

    def embed_read(self, embed_ids) -> np.ndarray:
        ids = _i32(embed_ids)
        t = torch.empty((len(ids), self.model.hidden), dtype=torch.bfloat16, device=self.device)
        torch.cuda.synchronize(self.device)
        self._check(self.lib.pie_embed_read(self.ctx, _ptr(ids), len(ids), C.c_void_p(t.data_ptr())))
        return t.view(torch.int16).cpu().numpy().view(np.uint16)

    def kv_write(self, layer: int, page_ids, slots, k_bits, v_bits, chunk: int = 1 << 16):
        p, s = _i32(page_ids), _i32(slots)
        k_bits = np.ascontiguousarray(k_bits, dtype=np.uint16)
        v_bits = np.ascontiguousarray(v_bits, dtype=np.uint16)
        for a in range(0, len(p), chunk):  # bounded staging copies
            b = min(len(p), a + chunk)
            k, v = self._dev_bf16(k_bits[a:b]), self._dev_bf16(v_bits[a:b])
            torch.cuda.synchronize(self.device)
            self._check(self.lib.pie_kv_write(self.ctx, layer, _ptr(p[a:b].copy()), _ptr(s[a:b].copy()), b - a,
                                              C.c_void_p(k.data_ptr()), C.c_void_p(v.data_ptr())))

    def mask_kvpage(self, page_ids, visible_bits):
        p = _i32(page_ids)
        bits = np.ascontiguousarray(visible_bits, dtype=np.uint32)
        if len(p) != len(bits):
            raise ValueError("mask_kvpage: one mask per page")
        self._check(self.lib.pie_mask_kvpage(self.ctx, _ptr(p), _ptr(bits), len(p)))

    def copy_kvpage(self, src_pages, src_slots, dst_pages, dst_slots):
        a = [_i32(x) for x in (src_pages, src_slots, dst_pages, dst_slots)]
        if len({len(x) for x in a}) != 1:
            raise ValueError("copy_kvpage: four arrays of one length")
        self._check(self.lib.pie_copy_kvpage(self.ctx, *[_ptr(x) for x in a], len(a[0])))

    def kv_read(self, layer: int, page_ids, slots):
        p, s = _i32(page_ids), _i32(slots)
        m = self.model
        k = torch.empty((len(p), m.n_kv_heads, m.head_dim), dtype=torch.bfloat16, device=self.device)
        v = torch.empty_like(k)
        torch.cuda.synchronize(self.device)
        self._check(self.lib.pie_kv_read(self.ctx, layer, _ptr(p), _ptr(s), len(p), C.c_void_p(k.data_ptr()),
                                         C.c_void_p(v.data_ptr())))
        f = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
        return f(k), f(v)

    # ---- forward ----
    def _batch_struct(self, b):
        arrs = dict(tok_indptr=_i32(b.tok_indptr), in_embed_ids=_i32(b.in_embed_ids),
                    out_embed_ids=_i32(b.out_embed_ids),
                    positions=None if b.positions is None else _i32(b.positions),
                    page_indptr=_i32(b.page_indptr), page_ids=_i32(b.page_ids), kv_len=_i32(b.kv_len))
        mi = None if b.mask_indptr is None else np.ascontiguousarray(b.mask_indptr, dtype=np.int64)
        mw = None if b.mask_words is None else np.ascontiguousarray(b.mask_words, dtype=np.uint32)
        ad = getattr(b, "adapter_ids", None)
        ad = None if ad is None else _i32(ad)
        fb = ForwardBatchC(int(b.n_requests), int(b.n_tokens), _ptr(arrs["tok_indptr"]), _ptr(arrs["in_embed_ids"]),
                           _ptr(arrs["out_embed_ids"]), _ptr(arrs["positions"]), _ptr(arrs["page_indptr"]),
                           _ptr(arrs["page_ids"]), _ptr(arrs["kv_len"]), _ptr(mi), _ptr(mw), _ptr(ad))
        return fb, (arrs, mi, mw, ad)

    def batch_create(self, batch, validate: bool = True) -> PieBatch:
        fb, keep = self._batch_struct(batch)
        h = C.c_void_p()
        self._check(self.lib.pie_batch_create(self.ctx, C.byref(fb), int(validate), C.byref(h)))
        return PieBatch(self, h, keep)

    def forward(self, layer: int, batch: PieBatch):
        self._check(self.lib.pie_forward(self.ctx, layer, batch.handle))

    def forward_all(self, batch: PieBatch):
        self._check(self.lib.pie_forward_all(self.ctx, batch.handle))

    def forward_host(self, layer: int, batch, validate: bool = True):
        fb, keep = self._batch_struct(batch)
        self._check(self.lib.pie_forward_host(self.ctx, layer, C.byref(fb), int(validate)))

    # ---- sample ----
    def get_next_dist_async(self, embed_ids, top_k: int, temperature: float, out_ids: torch.Tensor,
                            out_probs: torch.Tensor):
        ids = _i32(embed_ids)
        self._check(self.lib.pie_get_next_dist(self.ctx, _ptr(ids), len(ids), top_k, float(temperature),
                                               C.c_void_p(out_ids.data_ptr()), C.c_void_p(out_probs.data_ptr())))

    def get_next_dist_static_async(self, embed_ids, top_k: int, temperature: float, out_ids: torch.Tensor,
                                   out_probs: torch.Tensor):
        """pie_get_next_dist_static: the allocation-free variant (at most 16 rows); outputs are caller tensors."""
        ids = _i32(embed_ids)
        self._check(self.lib.pie_get_next_dist_static(self.ctx, _ptr(ids), len(ids), top_k, float(temperature),
                                                      C.c_void_p(out_ids.data_ptr()), C.c_void_p(out_probs.data_ptr())))

    def forward_dist(self, batch: PieBatch, rows, top_k: int, temperature: float = 1.0):
        r = _i32(rows)
        oi = torch.empty((len(r), top_k), dtype=torch.int32, device=self.device)
        op = torch.empty((len(r), top_k), dtype=torch.float32, device=self.device)
        torch.cuda.synchronize(self.device)
        self._check(self.lib.pie_forward_dist(self.ctx, batch.handle, _ptr(r), len(r), top_k, float(temperature),
                                              C.c_void_p(oi.data_ptr()), C.c_void_p(op.data_ptr())))
        self.synchronize()
        return oi.cpu().numpy(), op.cpu().numpy()

    def get_next_dist(self, embed_ids, top_k: int, temperature: float = 1.0):
        n = len(embed_ids)
        oi = torch.empty((n, top_k), dtype=torch.int32, device=self.device)
        op = torch.empty((n, top_k), dtype=torch.float32, device=self.device)
        torch.cuda.synchronize(self.device)
        self.get_next_dist_async(embed_ids, top_k, temperature, oi, op)
        self.synchronize()
        return oi.cpu().numpy(), op.cpu().numpy()

    def synchronize(self):
        self._check(self.lib.pie_synchronize(self.ctx))

    # ---- observation ----
    def read_tap(self, which: int, rows: int) -> np.ndarray:
        m = self.model
        if which in (TAP_Q, TAP_ATTN):
            shape, dt = (rows, m.n_q_heads * m.head_dim), torch.bfloat16
        elif which == TAP_RESID:
            shape, dt = (rows, m.hidden), torch.float32
        elif which == TAP_ACT:
            shape, dt = (rows, m.mlp_dim), torch.bfloat16
        else:
            shape, dt = (rows, m.vocab), torch.float32
        t = torch.empty(shape, dtype=dt, device=self.device)
        torch.cuda.synchronize(self.device)
        self._check(self.lib.pie_read_tap(self.ctx, which, C.c_void_p(t.data_ptr()), t.numel()))
        if dt == torch.bfloat16:
            return t.view(torch.int16).cpu().numpy().view(np.uint16)
        return t.cpu().numpy()

    def set_stage_timing(self, enabled: bool):
        self._check(self.lib.pie_set_stage_timing(self.ctx, int(enabled)))

    def stage_times(self) -> dict:
        out = np.zeros(PIE_N_STAGES, dtype=np.float32)
        self._check(self.lib.pie_stage_times(self.ctx, _ptr(out)))
        return {STAGE_NAMES[i]: float(out[i]) for i in range(PIE_N_STAGES)}
