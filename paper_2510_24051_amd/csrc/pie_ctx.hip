// C ABI of libpie_mi355: context, resource pools, batch deserialisation and the per-layer launch sequence.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <unordered_map>
#include <unordered_set>

#include "internal.h"

static char g_create_err[512] = "";

// Scratch memory of pie_get_next_dist_static, the entry point for callers that cannot allocate: one array per GPU,
// held until the process ends.  In host code `pie_static_scratch` is only a handle for hipGetSymbolAddress; the
// device address of each GPU's copy is looked up once per device in pie_create and kept in g_static_scratch.
#define PIE_STATIC_SCRATCH_BYTES (16u << 20)
#define PIE_STATIC_DIST_ROWS 32
#define PIE_MAX_DEVICES 64
static __device__ __align__(256) unsigned char pie_static_scratch[PIE_STATIC_SCRATCH_BYTES];
static void* g_static_scratch[PIE_MAX_DEVICES] = {nullptr};

static pie_status fail(pie_ctx* ctx, pie_status code, const char* fmt, ...) {
  char* dst = ctx ? ctx->err : g_create_err;
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(dst, 512, fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(ctx, expr)                                                                          \
  do {                                                                                              \
    hipError_t _e = (expr);                                                                         \
    if (_e != hipSuccess)                                                                           \
      return fail(ctx, _e == hipErrorOutOfMemory ? PIE_ENOMEM : PIE_EHIP, "%s: %s", #expr, hipGetErrorString(_e)); \
  } while (0)

extern "C" const char* pie_last_error(const pie_ctx* ctx) { return ctx ? ctx->err : g_create_err; }

// No C++ exception may cross the C boundary: entry points that build host containers run through this.
template <typename F>
static pie_status guarded(pie_ctx* ctx, const char* what, F&& body) {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return fail(ctx, PIE_ENOMEM, "%s: out of host memory", what);
  } catch (...) {
    return fail(ctx, PIE_EINVAL, "%s: unexpected exception", what);
  }
}

// ---------------------------------------------------------------------------------------------
// create / destroy
// ---------------------------------------------------------------------------------------------
template <typename T>
static hipError_t dev_alloc(T** p, size_t elems, bool zero, hipStream_t s) {
  *p = nullptr;
  if (elems == 0) return hipSuccess;
  hipError_t e = hipMalloc(reinterpret_cast<void**>(p), elems * sizeof(T));
  if (e != hipSuccess) return e;
  if (zero) e = hipMemsetAsync(*p, 0, elems * sizeof(T), s);
  return e;
}

static int round_up(int x, int m) { return (x + m - 1) / m * m; }

static pie_status pie_create_impl(const pie_model_desc* m, const pie_pool_desc* p, void* hip_stream, pie_ctx** out,
                                  int planner_wave_slots = 0) {
  if (!m || !p || !out) return fail(nullptr, PIE_EINVAL, "pie_create: null argument");
  *out = nullptr;
  if (m->page_size != PAGE && m->page_size != 2 * PAGE)
    return fail(nullptr, PIE_EUNSUPPORTED, "page_size %d: the kernels work on blocks of %d tokens and take pages of %d or %d", m->page_size, PAGE, PAGE, 2 * PAGE);
  const int F = m->page_size / PAGE;  // 16-token blocks per KvPage
  if (m->head_dim != 64 && m->head_dim != 128) return fail(nullptr, PIE_EUNSUPPORTED, "head_dim %d: need 64 or 128", m->head_dim);
  if (m->n_kv_heads <= 0 || m->n_q_heads % m->n_kv_heads != 0 || m->n_q_heads / m->n_kv_heads > 8)
    return fail(nullptr, PIE_EUNSUPPORTED, "need n_q_heads = group * n_kv_heads with group <= 8");
  if (m->hidden <= 0 || m->hidden % 32 || m->mlp_dim <= 0 || m->mlp_dim % 32 || m->vocab < 0 || m->vocab % 32 ||
      m->hidden > 8192)
    return fail(nullptr, PIE_EUNSUPPORTED, "hidden (<= 8192), mlp_dim and vocab must be multiples of 32");
  if (m->vocab > 0 && topk_chunks(m->vocab, 1) == 0)
    return fail(nullptr, PIE_EUNSUPPORTED, "vocab %d: the top-k kernels handle up to 131072 entries", m->vocab);
  if (m->n_layers <= 0 || !(m->rms_eps > 0.f) || !(m->rope_theta > 0.f))
    return fail(nullptr, PIE_EINVAL, "n_layers, rms_eps and rope_theta must be positive");
  if (p->n_kv_pages <= 0 || p->n_embeds <= 0 || p->max_batch_tokens <= 0 || p->max_batch_requests <= 0 ||
      p->max_top_k < 0 || p->max_dist_rows < 0 || p->max_top_k > 1024)
    return fail(nullptr, PIE_EINVAL, "pool sizes must be positive (max_top_k <= 1024)");
  if (p->max_adapters < 0 || p->max_lora_rank < 0 || (p->max_adapters > 0) != (p->max_lora_rank > 0) ||
      p->max_lora_rank > 1024)
    return fail(nullptr, PIE_EINVAL, "max_adapters and max_lora_rank (<= 1024) must both be 0 or both be positive");
  if ((int64_t)p->n_kv_pages * F * m->n_kv_heads > INT32_MAX)
    return fail(nullptr, PIE_EUNSUPPORTED, "n_kv_pages * n_kv_heads must fit 31 bits (page-head block indices are int32)");

  pie_ctx* c = new pie_ctx();
  c->m = *m;
  c->p = *p;
  c->stream = reinterpret_cast<hipStream_t>(hip_stream);
  c->err[0] = 0;
  for (int i = 0; i < PIE_N_STAGES; ++i) c->ev_used[i] = false;
  for (int i = 0; i < 2 * PIE_N_STAGES; ++i) c->ev[i] = nullptr;
  if (planner_wave_slots > 0) {  // host-only context: deserialisation and planning, nothing on a device
    c->host_only = true;
    c->wave_slots = planner_wave_slots;
    c->layers.resize(m->n_layers);
    c->embed_pos.assign((size_t)p->n_embeds, -1);
    c->page_mask.assign((size_t)p->n_kv_pages * F, 0xFFFFu);
    c->blocks_per_page = F;
    if (p->max_adapters > 0) c->lora.assign((size_t)p->max_adapters * m->n_layers * PIE_N_PROJ, LoraPair());
    *out = c;
    return PIE_OK;
  }
  hipError_t e = hipGetDevice(&c->device);
  if (e == hipSuccess && c->device >= 0 && c->device < PIE_MAX_DEVICES) {
    // this GPU's copy of the static scratch array (the context's device is current here)
    if (!g_static_scratch[c->device]) {
      void* ptr = nullptr;
      e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(pie_static_scratch));
      if (e == hipSuccess) g_static_scratch[c->device] = ptr;
    }
    c->static_scratch = reinterpret_cast<unsigned char*>(g_static_scratch[c->device]);
  }
  {
    int cus = 0;
    if (e == hipSuccess && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) == hipSuccess && cus > 0)
      c->wave_slots = cus * 8;  // the decode kernel runs two waves per SIMD
  }
  const int H = m->hidden, QD = m->n_q_heads * m->head_dim, KD = m->n_kv_heads * m->head_dim, I = m->mlp_dim;
  const size_t T = (size_t)p->max_batch_tokens;
  c->layers.resize(m->n_layers);
  c->blocks_per_page = F;
  c->kv_layer_elems = (size_t)p->n_kv_pages * F * m->n_kv_heads * 2 * PAGE * m->head_dim;
  auto chk = [&](hipError_t x) { if (e == hipSuccess) e = x; };
  chk(dev_alloc(&c->embeds, (size_t)p->n_embeds * H, true, c->stream));
  chk(dev_alloc(&c->kv, c->kv_layer_elems * m->n_layers, true, c->stream));
  chk(dev_alloc(&c->xn, T * H, false, c->stream));
  chk(dev_alloc(&c->qkv, T * (QD + 2 * KD), false, c->stream));
  chk(dev_alloc(&c->attn, T * QD, false, c->stream));
  chk(dev_alloc(&c->h, T * H, false, c->stream));
  if (m->n_layers > 1) chk(dev_alloc(&c->x32, T * H, false, c->stream));
  if (p->max_adapters > 0) {
    c->lora.assign((size_t)p->max_adapters * m->n_layers * PIE_N_PROJ, LoraPair());
    chk(dev_alloc(&c->lora_dev, c->lora.size(), true, c->stream));
    // rows: every token once, each adapter's group padded to whole tiles of 32; at least 2048 so that small
    // batches can split the input dimension over workgroups (partial copies)
    c->lora_z_rows = std::max<size_t>(T + 32 * (size_t)p->max_adapters, 2048);
    chk(dev_alloc(&c->lora_z, c->lora_z_rows * 3 * round_up(p->max_lora_rank, 16), false, c->stream));
  }
  c->embed_pos.assign((size_t)p->n_embeds, -1);
  c->page_mask.assign((size_t)p->n_kv_pages * F, 0xFFFFu);
  chk(dev_alloc(&c->act, T * I, false, c->stream));
  // split-K workspace: only batches of <= 256 rows use it; 8 partial copies of the widest output
  {
    size_t rows = std::min<size_t>(std::max<size_t>(T, (size_t)p->max_dist_rows), 256);
    size_t widest = std::max<size_t>((size_t)2 * I, (size_t)round_up(std::max(QD + 2 * KD, H), 32));
    c->splitk_elems = rows * widest * 8;
    chk(dev_alloc(&c->splitk, c->splitk_elems, false, c->stream));
  }
  if (m->vocab > 0 && p->max_dist_rows > 0) {
    chk(dev_alloc(&c->logits, (size_t)p->max_dist_rows * m->vocab, false, c->stream));
    chk(dev_alloc(&c->en, (size_t)p->max_dist_rows * H, false, c->stream));
    chk(dev_alloc(&c->topk_cand, (size_t)p->max_dist_rows * 16 * std::max(p->max_top_k, 1), false, c->stream));
    chk(dev_alloc(&c->topk_stats, (size_t)p->max_dist_rows * 16 * 2, false, c->stream));
  }
  // staging for id lists: get_next_dist stages at most max_dist_rows ids, so the serving path never outgrows it
  // (only the seeding / inspection calls may, and they re-allocate)
  c->ids_cap = std::max<size_t>(std::max<size_t>(4096, 2 * T), (size_t)p->max_dist_rows);
  chk(dev_alloc(&c->ids_dev, c->ids_cap, false, c->stream));
  chk(dev_alloc(&c->inv_freq, (size_t)m->head_dim / 2, false, c->stream));
  if (e == hipSuccess) {
    std::vector<double> f(m->head_dim / 2);
    for (int i = 0; i < m->head_dim / 2; ++i) f[i] = std::pow((double)m->rope_theta, -2.0 * i / m->head_dim);
    chk(hipMemcpyAsync(c->inv_freq, f.data(), f.size() * sizeof(double), hipMemcpyHostToDevice, c->stream));
    chk(hipStreamSynchronize(c->stream));
  }
  for (int i = 0; i < 2 * PIE_N_STAGES && e == hipSuccess; ++i) chk(hipEventCreate(&c->ev[i]));
  if (e != hipSuccess) {
    pie_status st = fail(nullptr, e == hipErrorOutOfMemory ? PIE_ENOMEM : PIE_EHIP, "pie_create: %s", hipGetErrorString(e));
    pie_destroy(c);
    return st;
  }
  *out = c;
  return PIE_OK;
}

extern "C" pie_status pie_create(const pie_model_desc* m, const pie_pool_desc* p, void* hip_stream, pie_ctx** out) {
  return guarded(nullptr, "pie_create", [&]() { return pie_create_impl(m, p, hip_stream, out); });
}

extern "C" pie_status pie_create_planner(const pie_model_desc* m, const pie_pool_desc* p, int32_t wave_slots,
                                         pie_ctx** out) {
  if (wave_slots <= 0 || wave_slots % 8 != 0)
    return fail(nullptr, PIE_EINVAL, "pie_create_planner: wave_slots must be a positive multiple of 8");
  return guarded(nullptr, "pie_create_planner", [&]() { return pie_create_impl(m, p, nullptr, out, wave_slots); });
}

static void free_packed(PackedWeight& w) {
  if (w.data) (void)hipFree(w.data);
  w = PackedWeight();
}

extern "C" pie_status pie_destroy(pie_ctx* c) {
  if (!c) return PIE_OK;
  if (c->host_only) {  // nothing lives on a device
    std::free(c->host_blob);
    delete c;
    return PIE_OK;
  }
  (void)hipStreamSynchronize(c->stream);
  for (auto& L : c->layers) {
    if (L.g1) (void)hipFree(L.g1);
    if (L.g2) (void)hipFree(L.g2);
    free_packed(L.wqkv); free_packed(L.wo); free_packed(L.wgu); free_packed(L.wdown);
  }
  free_packed(c->wlm);
  void* bufs[] = {c->embeds, c->kv, c->xn, c->qkv, c->attn, c->h, c->act, c->splitk, c->logits, c->en,
                  c->ids_dev, c->inv_freq, c->g_final, c->topk_cand, c->topk_stats, c->table, c->x32, c->lora_dev, c->lora_z, c->gu32};
  for (LoraPair& lp : c->lora) {
    if (lp.A) (void)hipFree(lp.A);
    if (lp.B) (void)hipFree(lp.B);
  }
  for (void* b : bufs) if (b) (void)hipFree(b);
  for (auto& blk : c->blob_pool) (void)hipFree(blk.first);
  if (c->host_blob) { if (c->host_blob_pinned) (void)hipHostFree(c->host_blob); else std::free(c->host_blob); }
  for (int i = 0; i < 2 * PIE_N_STAGES; ++i) if (c->ev[i]) (void)hipEventDestroy(c->ev[i]);
  delete c;
  return PIE_OK;
}

// ---------------------------------------------------------------------------------------------
// weights
// ---------------------------------------------------------------------------------------------
static pie_status pack_into(pie_ctx* c, PackedWeight& w, int N, int K, const void* s0, int r0, const void* s1, int r1,
                            const void* s2, int r2, int interleave) {
  free_packed(w);
  w.N = N;
  w.K = K;
  w.NB = (N + 31) / 32;
  HIP_TRY(c, hipMalloc(reinterpret_cast<void**>(&w.data), (size_t)w.NB * 32 * K * sizeof(bf16_t)));
  HIP_TRY(c, launch_pack_weight((const bf16_t*)s0, r0, (const bf16_t*)s1, r1, (const bf16_t*)s2, r2, K, interleave,
                                w.data, w.NB, c->stream));
  return PIE_OK;
}

static pie_status copy_gain(pie_ctx* c, bf16_t** dst, const void* src, int H) {
  if (!*dst) HIP_TRY(c, hipMalloc(reinterpret_cast<void**>(dst), (size_t)H * sizeof(bf16_t)));
  HIP_TRY(c, hipMemcpyAsync(*dst, src, (size_t)H * sizeof(bf16_t), hipMemcpyDeviceToDevice, c->stream));
  return PIE_OK;
}

extern "C" pie_status pie_load_layer(pie_ctx* c, int32_t layer, const void* g1, const void* wq, const void* wk,
                                     const void* wv, const void* wo, const void* g2, const void* wgate,
                                     const void* wup, const void* wdown) {
  if (!c) return PIE_EINVAL;
  if (c->host_only) return fail(c, PIE_EINVAL, "pie_load_layer: the context only plans batches (pie_create_planner)");
  if (!g1 || !wq || !wk || !wv || !wo || !g2 || !wgate || !wup || !wdown) return fail(c, PIE_EINVAL, "pie_load_layer: null weight");
  if (layer < 0 || layer >= c->m.n_layers) return fail(c, PIE_ERANGE, "pie_load_layer: layer %d of %d", layer, c->m.n_layers);
  const int H = c->m.hidden, QD = c->m.n_q_heads * c->m.head_dim, KD = c->m.n_kv_heads * c->m.head_dim, I = c->m.mlp_dim;
  LayerWeights& L = c->layers[layer];
  L.loaded = false;
  pie_status st;
  if ((st = copy_gain(c, &L.g1, g1, H)) != PIE_OK) return st;
  if ((st = copy_gain(c, &L.g2, g2, H)) != PIE_OK) return st;
  if ((st = pack_into(c, L.wqkv, QD + 2 * KD, H, wq, QD, wk, KD, wv, KD, 0)) != PIE_OK) return st;
  if ((st = pack_into(c, L.wo, H, QD, wo, H, nullptr, 0, nullptr, 0, 0)) != PIE_OK) return st;
  if ((st = pack_into(c, L.wgu, 2 * I, H, wgate, I, wup, I, nullptr, 0, 1)) != PIE_OK) return st;
  if ((st = pack_into(c, L.wdown, H, I, wdown, H, nullptr, 0, nullptr, 0, 0)) != PIE_OK) return st;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  L.loaded = true;
  return PIE_OK;
}

extern "C" pie_status pie_load_head(pie_ctx* c, const void* g_final, const void* w_lm) {
  if (!c) return PIE_EINVAL;
  if (c->host_only) return fail(c, PIE_EINVAL, "pie_load_head: the context only plans batches (pie_create_planner)");
  if (!w_lm) return fail(c, PIE_EINVAL, "pie_load_head: null weight");
  if (c->m.vocab <= 0 || !c->logits) return fail(c, PIE_EINVAL, "pie_load_head: context created without vocab / dist rows");
  c->head_loaded = false;
  pie_status st;
  if (g_final) {
    if ((st = copy_gain(c, &c->g_final, g_final, c->m.hidden)) != PIE_OK) return st;
  } else if (c->g_final) {
    (void)hipFree(c->g_final);
    c->g_final = nullptr;
  }
  if ((st = pack_into(c, c->wlm, c->m.vocab, c->m.hidden, w_lm, c->m.vocab, nullptr, 0, nullptr, 0, 0)) != PIE_OK) return st;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  c->head_loaded = true;
  return PIE_OK;
}

extern "C" pie_status pie_load_embedding(pie_ctx* c, const void* table) {
  if (!c) return PIE_EINVAL;
  if (c->host_only) return fail(c, PIE_EINVAL, "pie_load_embedding: the context only plans batches (pie_create_planner)");
  if (!table) return fail(c, PIE_EINVAL, "pie_load_embedding: null table");
  if (c->m.vocab <= 0) return fail(c, PIE_EINVAL, "pie_load_embedding: context created without vocab");
  const size_t bytes = (size_t)c->m.vocab * c->m.hidden * sizeof(bf16_t);
  if (!c->table) {
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&c->table), bytes);
    if (e != hipSuccess) return fail(c, e == hipErrorOutOfMemory ? PIE_ENOMEM : PIE_EHIP, "pie_load_embedding: %s", hipGetErrorString(e));
  }
  HIP_TRY(c, hipMemcpyAsync(c->table, table, bytes, hipMemcpyDeviceToDevice, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return PIE_OK;
}

extern "C" pie_status pie_load_adapter(pie_ctx* c, int32_t adapter, int32_t layer, int32_t proj, int32_t rank,
                                       float scale, const void* A, const void* B) {
  if (!c) return PIE_EINVAL;
  if (c->host_only) return fail(c, PIE_EINVAL, "pie_load_adapter: the context only plans batches (pie_create_planner)");
  if (c->p.max_adapters <= 0) return fail(c, PIE_EINVAL, "pie_load_adapter: context created without adapters");
  if (adapter < 0 || adapter >= c->p.max_adapters) return fail(c, PIE_ERANGE, "adapter %d outside [0, %d)", adapter, c->p.max_adapters);
  if (layer < 0 || layer >= c->m.n_layers) return fail(c, PIE_ERANGE, "layer %d of %d", layer, c->m.n_layers);
  if (proj < 0 || proj >= PIE_N_PROJ) return fail(c, PIE_ERANGE, "projection %d outside [0, %d)", proj, PIE_N_PROJ);
  if (rank < 0 || rank > c->p.max_lora_rank) return fail(c, PIE_ERANGE, "rank %d outside [0, %d]", rank, c->p.max_lora_rank);
  if (rank > 0 && (!A || !B)) return fail(c, PIE_EINVAL, "pie_load_adapter: null pair with rank %d", rank);
  if (!std::isfinite(scale)) return fail(c, PIE_EINVAL, "pie_load_adapter: scale must be finite");
  const pie_model_desc& m = c->m;
  const int QD = m.n_q_heads * m.head_dim, KD = m.n_kv_heads * m.head_dim;
  const int outs[PIE_N_PROJ] = {QD, KD, KD, m.hidden, m.mlp_dim, m.mlp_dim, m.hidden};
  const int ins[PIE_N_PROJ] = {m.hidden, m.hidden, m.hidden, QD, m.hidden, m.hidden, m.mlp_dim};
  HIP_TRY(c, hipStreamSynchronize(c->stream));  // no kernel may still read the pair that is replaced
  LoraPair& lp = c->lora[((size_t)adapter * m.n_layers + layer) * PIE_N_PROJ + proj];
  if (lp.A) (void)hipFree(lp.A);
  if (lp.B) (void)hipFree(lp.B);
  lp = LoraPair();
  if (rank > 0 && A && B) {
    const int rank_p = round_up(rank, 16);
    const size_t a_bytes = (size_t)rank_p * ins[proj] * sizeof(bf16_t), b_bytes = (size_t)outs[proj] * rank_p * sizeof(bf16_t);
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&lp.A), a_bytes);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&lp.B), b_bytes);
    if (e != hipSuccess) {
      if (lp.A) (void)hipFree(lp.A);
      lp = LoraPair();
      return fail(c, e == hipErrorOutOfMemory ? PIE_ENOMEM : PIE_EHIP, "pie_load_adapter: %s", hipGetErrorString(e));
    }
    // zero padding: rows rank .. rank_p of A, columns rank .. rank_p of every row of B
    HIP_TRY(c, hipMemsetAsync(lp.A, 0, a_bytes, c->stream));
    HIP_TRY(c, hipMemsetAsync(lp.B, 0, b_bytes, c->stream));
    HIP_TRY(c, hipMemcpyAsync(lp.A, A, (size_t)rank * ins[proj] * sizeof(bf16_t), hipMemcpyDeviceToDevice, c->stream));
    HIP_TRY(c, hipMemcpy2DAsync(lp.B, (size_t)rank_p * sizeof(bf16_t), B, (size_t)rank * sizeof(bf16_t),
                                (size_t)rank * sizeof(bf16_t), (size_t)outs[proj], hipMemcpyDeviceToDevice, c->stream));
    lp.rank_p = rank_p;
    lp.rank = rank;
    lp.scale = scale;
    if ((proj == PIE_PROJ_GATE || proj == PIE_PROJ_UP) && !c->gu32) {
      // adapted gate/up: the SwiGLU product is taken from fp32 sums instead of the GEMM epilogue
      hipError_t e2 = hipMalloc(reinterpret_cast<void**>(&c->gu32), (size_t)c->p.max_batch_tokens * 2 * m.mlp_dim * sizeof(float));
      if (e2 != hipSuccess) {
        (void)hipFree(lp.A); (void)hipFree(lp.B);
        lp = LoraPair();
        return fail(c, e2 == hipErrorOutOfMemory ? PIE_ENOMEM : PIE_EHIP, "pie_load_adapter: %s", hipGetErrorString(e2));
      }
    }
  }
  HIP_TRY(c, hipMemcpyAsync(c->lora_dev, c->lora.data(), c->lora.size() * sizeof(LoraPair), hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return PIE_OK;
}

// ---------------------------------------------------------------------------------------------
// resource seeding / inspection
// ---------------------------------------------------------------------------------------------
static pie_status stage_ids(pie_ctx* c, const int32_t* a, const int32_t* b, int n) {
  if ((size_t)n * (b ? 2 : 1) > c->ids_cap) {
    (void)hipStreamSynchronize(c->stream);
    if (c->ids_dev) (void)hipFree(c->ids_dev);
    c->ids_dev = nullptr;
    c->ids_cap = (size_t)n * 2;
    HIP_TRY(c, hipMalloc(reinterpret_cast<void**>(&c->ids_dev), c->ids_cap * sizeof(int32_t)));
  }
  HIP_TRY(c, hipMemcpyAsync(c->ids_dev, a, (size_t)n * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
  if (b) HIP_TRY(c, hipMemcpyAsync(c->ids_dev + n, b, (size_t)n * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
  return PIE_OK;
}

static pie_status embed_copy(pie_ctx* c, const int32_t* ids, int32_t n, void* buf, int to_pool) {
  if (!c) return PIE_EINVAL;
  if (c->host_only) return fail(c, PIE_EINVAL, "pie_embed_write / pie_embed_read: the context only plans batches (pie_create_planner)");
  if (n < 0 || (n > 0 && (!ids || !buf))) return fail(c, PIE_EINVAL, "embed copy: null argument");
  if (n == 0) return PIE_OK;
  for (int i = 0; i < n; ++i)
    if (ids[i] < 0 || ids[i] >= c->p.n_embeds) return fail(c, PIE_ERANGE, "embed id %d at %d outside [0, %d)", ids[i], i, c->p.n_embeds);
  pie_status st = stage_ids(c, ids, nullptr, n);
  if (st != PIE_OK) return st;
  HIP_TRY(c, launch_embed_copy(c->embeds, c->ids_dev, n, c->m.hidden, (bf16_t*)buf, to_pool, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));  // ids_dev is reused by the next call
  return PIE_OK;
}
extern "C" pie_status pie_embed_write(pie_ctx* c, const int32_t* ids, int32_t n, const void* src) {
  pie_status st = embed_copy(c, ids, n, const_cast<void*>(src), 1);
  if (st == PIE_OK)
    for (int i = 0; i < n; ++i) c->embed_pos[ids[i]] = -1;  // raw contents carry no sequence position
  return st;
}

static pie_status pie_embed_txt_impl(pie_ctx* c, const int32_t* token_ids, const int32_t* positions, int32_t n,
                                    const int32_t* embed_ids) {
  if (!c) return PIE_EINVAL;
  if (c->host_only) return fail(c, PIE_EINVAL, "pie_embed_txt: the context only plans batches (pie_create_planner)");
  if (n < 0 || (n > 0 && (!token_ids || !positions || !embed_ids))) return fail(c, PIE_EINVAL, "pie_embed_txt: null argument");
  if (!c->table) return fail(c, PIE_EINVAL, "pie_embed_txt: no embedding table loaded");
  if (n == 0) return PIE_OK;
  std::unordered_set<int32_t> seen;
  seen.reserve((size_t)n * 2);
  for (int i = 0; i < n; ++i) {
    if (token_ids[i] < 0 || token_ids[i] >= c->m.vocab)
      return fail(c, PIE_ERANGE, "token id %d at %d outside [0, %d)", token_ids[i], i, c->m.vocab);
    if (embed_ids[i] < 0 || embed_ids[i] >= c->p.n_embeds)
      return fail(c, PIE_ERANGE, "embed id %d at %d outside [0, %d)", embed_ids[i], i, c->p.n_embeds);
    if (positions[i] < 0) return fail(c, PIE_ERANGE, "negative position %d at %d", positions[i], i);
    if (!seen.insert(embed_ids[i]).second)
      return fail(c, PIE_ECONFLICT, "embed id %d is written twice by one embed_txt call", embed_ids[i]);
  }
  pie_status st = stage_ids(c, embed_ids, token_ids, n);
  if (st != PIE_OK) return st;
  HIP_TRY(c, launch_embed_gather(c->embeds, c->ids_dev, c->ids_dev + n, n, c->m.hidden, c->table, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));  // ids_dev is reused by the next call
  for (int i = 0; i < n; ++i) c->embed_pos[embed_ids[i]] = positions[i];
  return PIE_OK;
}

extern "C" pie_status pie_embed_txt(pie_ctx* c, const int32_t* token_ids, const int32_t* positions, int32_t n,
                                    const int32_t* embed_ids) {
  return guarded(c, "pie_embed_txt", [&]() { return pie_embed_txt_impl(c, token_ids, positions, n, embed_ids); });
}
extern "C" pie_status pie_embed_read(pie_ctx* c, const int32_t* ids, int32_t n, void* dst) {
  return embed_copy(c, ids, n, dst, 0);
}

// KvPages of 2 x 16 tokens are stored as two consecutive 16-token blocks: page p, slot s -> block 2p + s / 16, slot s % 16.
static void to_blocks(const pie_ctx* c, const int32_t* pages, const int32_t* slots, int n, std::vector<int32_t>& bp,
                      std::vector<int32_t>& bs) {
  bp.resize(n);
  bs.resize(n);
  for (int i = 0; i < n; ++i) {
    bp[i] = pages[i] * c->blocks_per_page + slots[i] / PAGE;
    bs[i] = slots[i] % PAGE;
  }
}

static pie_status kv_copy(pie_ctx* c, int32_t layer, const int32_t* pages, const int32_t* slots, int32_t n, void* k,
                          void* v, int to_pool) {
  if (!c) return PIE_EINVAL;
  if (c->host_only) return fail(c, PIE_EINVAL, "pie_kv_write / pie_kv_read: the context only plans batches (pie_create_planner)");
  if (n < 0 || (n > 0 && (!pages || !slots || !k || !v))) return fail(c, PIE_EINVAL, "kv copy: null argument");
  if (layer < 0 || layer >= c->m.n_layers) return fail(c, PIE_ERANGE, "kv copy: layer %d of %d", layer, c->m.n_layers);
  if (n == 0) return PIE_OK;
  for (int i = 0; i < n; ++i) {
    if (pages[i] < 0 || pages[i] >= c->p.n_kv_pages) return fail(c, PIE_ERANGE, "page id %d at %d outside [0, %d)", pages[i], i, c->p.n_kv_pages);
    if (slots[i] < 0 || slots[i] >= c->m.page_size) return fail(c, PIE_ERANGE, "slot %d at %d outside [0, %d)", slots[i], i, c->m.page_size);
  }
  std::vector<int32_t> bp, bs;  // pages of two 16-token blocks: (page, slot) -> (block, slot within the block)
  if (c->blocks_per_page > 1) {
    to_blocks(c, pages, slots, n, bp, bs);
    pages = bp.data();
    slots = bs.data();
  }
  pie_status st = stage_ids(c, pages, slots, n);
  if (st != PIE_OK) return st;
  HIP_TRY(c, launch_kv_copy(c->kv + (size_t)layer * c->kv_layer_elems, c->ids_dev, c->ids_dev + n, n, c->m.n_kv_heads,
                            c->m.head_dim, (bf16_t*)k, (bf16_t*)v, to_pool, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return PIE_OK;
}
extern "C" pie_status pie_kv_write(pie_ctx* c, int32_t layer, const int32_t* pages, const int32_t* slots, int32_t n,
                                   const void* k, const void* v) {
  return guarded(c, "pie_kv_write", [&]() { return kv_copy(c, layer, pages, slots, n, const_cast<void*>(k), const_cast<void*>(v), 1); });
}
extern "C" pie_status pie_kv_read(pie_ctx* c, int32_t layer, const int32_t* pages, const int32_t* slots, int32_t n,
                                  void* k, void* v) {
  return guarded(c, "pie_kv_read", [&]() { return kv_copy(c, layer, pages, slots, n, k, v, 0); });
}

extern "C" pie_status pie_mask_kvpage(pie_ctx* c, const int32_t* page_ids, const uint32_t* visible_bits, int32_t n) {
  if (!c) return PIE_EINVAL;
  if (n < 0 || (n > 0 && (!page_ids || !visible_bits))) return fail(c, PIE_EINVAL, "pie_mask_kvpage: null argument");
  for (int i = 0; i < n; ++i)
    if (page_ids[i] < 0 || page_ids[i] >= c->p.n_kv_pages)
      return fail(c, PIE_ERANGE, "page id %d at %d outside [0, %d)", page_ids[i], i, c->p.n_kv_pages);
  const int F = c->blocks_per_page;
  for (int i = 0; i < n; ++i)
    for (int f = 0; f < F; ++f) c->page_mask[(size_t)page_ids[i] * F + f] = (uint16_t)((visible_bits[i] >> (PAGE * f)) & 0xFFFFu);
  return PIE_OK;
}

static pie_status pie_copy_kvpage_impl(pie_ctx* c, const int32_t* src_pages, const int32_t* src_slots,
                                      const int32_t* dst_pages, const int32_t* dst_slots, int32_t n) {
  if (!c) return PIE_EINVAL;
  if (c->host_only) return fail(c, PIE_EINVAL, "pie_copy_kvpage: the context only plans batches (pie_create_planner)");
  if (n < 0 || (n > 0 && (!src_pages || !src_slots || !dst_pages || !dst_slots)))
    return fail(c, PIE_EINVAL, "pie_copy_kvpage: null argument");
  if (n == 0) return PIE_OK;
  const int PS = c->m.page_size;
  std::unordered_set<int64_t> src, dst;
  src.reserve((size_t)n * 2);
  dst.reserve((size_t)n * 2);
  for (int i = 0; i < n; ++i) {
    if (src_pages[i] < 0 || src_pages[i] >= c->p.n_kv_pages || dst_pages[i] < 0 || dst_pages[i] >= c->p.n_kv_pages)
      return fail(c, PIE_ERANGE, "page id at %d outside [0, %d)", i, c->p.n_kv_pages);
    if (src_slots[i] < 0 || src_slots[i] >= PS || dst_slots[i] < 0 || dst_slots[i] >= PS)
      return fail(c, PIE_ERANGE, "slot at %d outside [0, %d)", i, PS);
    src.insert((int64_t)src_pages[i] * PS + src_slots[i]);
    if (!dst.insert((int64_t)dst_pages[i] * PS + dst_slots[i]).second)
      return fail(c, PIE_ECONFLICT, "token (page %d, slot %d) is written twice by one copy", dst_pages[i], dst_slots[i]);
  }
  for (int64_t t : dst)
    if (src.count(t)) return fail(c, PIE_ECONFLICT, "token (page %lld, slot %lld) is both read and written by one copy",
                                  (long long)(t / PS), (long long)(t % PS));
  std::vector<int32_t> sbp, sbs, dbp, dbs;
  if (c->blocks_per_page > 1) {
    to_blocks(c, src_pages, src_slots, n, sbp, sbs);
    to_blocks(c, dst_pages, dst_slots, n, dbp, dbs);
    src_pages = sbp.data(); src_slots = sbs.data(); dst_pages = dbp.data(); dst_slots = dbs.data();
  }
  const int32_t* arrs[4] = {src_pages, src_slots, dst_pages, dst_slots};
  if ((size_t)n * 4 > c->ids_cap) {
    (void)hipStreamSynchronize(c->stream);
    if (c->ids_dev) (void)hipFree(c->ids_dev);
    c->ids_dev = nullptr;
    c->ids_cap = (size_t)n * 4;
    HIP_TRY(c, hipMalloc(reinterpret_cast<void**>(&c->ids_dev), c->ids_cap * sizeof(int32_t)));
  }
  for (int k = 0; k < 4; ++k)
    HIP_TRY(c, hipMemcpyAsync(c->ids_dev + (size_t)k * n, arrs[k], (size_t)n * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
  HIP_TRY(c, launch_kv_token_copy(c->kv, c->kv_layer_elems, c->m.n_layers, c->ids_dev, c->ids_dev + n, c->ids_dev + 2 * (size_t)n,
                                  c->ids_dev + 3 * (size_t)n, n, c->m.n_kv_heads, c->m.head_dim, c->stream));
  HIP_TRY(c, hipStreamSynchronize(c->stream));  // ids_dev is reused by the next call
  return PIE_OK;
}

extern "C" pie_status pie_copy_kvpage(pie_ctx* c, const int32_t* src_pages, const int32_t* src_slots,
                                      const int32_t* dst_pages, const int32_t* dst_slots, int32_t n) {
  return guarded(c, "pie_copy_kvpage", [&]() { return pie_copy_kvpage_impl(c, src_pages, src_slots, dst_pages, dst_slots, n); });
}

// ---------------------------------------------------------------------------------------------
// batch deserialisation
// ---------------------------------------------------------------------------------------------
namespace {
struct Blob {  // host image of the device allocation, written into the context's reusable buffer
  pie_ctx* c;
  size_t size = 0;
  bool ok = true;
  explicit Blob(pie_ctx* ctx) : c(ctx) {}
  unsigned char* data() const { return c->host_blob; }
  void reserve(size_t n) {
    if (n <= c->host_blob_cap) return;
    size_t cap = std::max<size_t>(std::max(n, c->host_blob_cap * 2), (size_t)1 << 20);
    unsigned char* p = nullptr;
    bool pinned = false;
    if (!c->host_only) {
      if (hipHostMalloc((void**)&p, cap, hipHostMallocDefault) == hipSuccess) pinned = true;
      else { (void)hipGetLastError(); p = nullptr; }
    }
    if (!p) p = (unsigned char*)std::malloc(cap);
    if (!p) { ok = false; return; }
    if (size) std::memcpy(p, c->host_blob, size);
    if (c->host_blob) { if (c->host_blob_pinned) (void)hipHostFree(c->host_blob); else std::free(c->host_blob); }
    c->host_blob = p; c->host_blob_cap = cap; c->host_blob_pinned = pinned;
  }
  void append(const void* src, size_t n) {  // n bytes from src (zeros when src is null), no alignment
    reserve(size + n);
    if (!ok || !n) return;
    if (src) std::memcpy(c->host_blob + size, src, n); else std::memset(c->host_blob + size, 0, n);
    size += n;
  }
  size_t add(const void* src, size_t n, size_t pad = 0) {  // at the next multiple of 256; pad zero bytes after
    const size_t off = (size + 255) / 256 * 256;
    reserve(off + n + pad);
    if (!ok) return off;
    std::memset(c->host_blob + size, 0, off - size);
    size = off;
    append(n ? src : nullptr, n);
    append(nullptr, pad);
    return off;
  }
};
}  // namespace

static pie_status pie_batch_create_impl(pie_ctx* c, const pie_forward_batch* b, int32_t validate, pie_batch** out) {
  if (!c) return PIE_EINVAL;
  if (!b || !out) return fail(c, PIE_EINVAL, "pie_batch_create: null argument");
  *out = nullptr;
  const int R = b->n_requests, T = b->n_tokens;
  if (R <= 0 || T <= 0) return fail(c, PIE_EINVAL, "empty batch (R=%d, T=%d)", R, T);
  if (R > c->p.max_batch_requests || T > c->p.max_batch_tokens)
    return fail(c, PIE_EBATCH, "batch of %d requests / %d tokens exceeds the context's %d / %d", R, T,
                c->p.max_batch_requests, c->p.max_batch_tokens);
  if (!b->tok_indptr || !b->in_embed_ids || !b->out_embed_ids || !b->page_indptr || !b->page_ids || !b->kv_len)
    return fail(c, PIE_EINVAL, "pie_batch_create: null array");
  if (b->mask_indptr && !b->mask_words && b->mask_indptr[R] > 0) return fail(c, PIE_EINVAL, "mask_indptr without mask_words");
  const int G = c->m.n_q_heads / c->m.n_kv_heads, Hkv = c->m.n_kv_heads, D = c->m.head_dim;
  if (b->tok_indptr[0] != 0 || b->tok_indptr[R] != T) return fail(c, PIE_EINVAL, "tok_indptr must run from 0 to n_tokens");
  if (b->page_indptr[0] != 0) return fail(c, PIE_EINVAL, "page_indptr must start at 0");

  // KvPages of 32 tokens are two consecutive 16-token blocks of the pool: the page tables are rewritten in blocks
  // (page p -> blocks 2p, 2p + 1) and everything below, like the kernels, works on 16-token blocks.
  const int F = c->blocks_per_page;
  const int n_pool_blocks = c->p.n_kv_pages * F;
  std::vector<int32_t> blk_indptr, blk_ids;
  pie_forward_batch in_blocks;
  if (F > 1) {
    blk_indptr.assign(R + 1, 0);
    for (int r = 0; r < R; ++r) {
      const int p0 = b->page_indptr[r], p1 = b->page_indptr[r + 1];
      if (p1 < p0) return fail(c, PIE_EINVAL, "bad page_indptr");
      const int need = (b->kv_len[r] + c->m.page_size - 1) / c->m.page_size;
      if (p1 - p0 < need) return fail(c, PIE_EINVAL, "request %d: %d pages listed, kv_len %d needs %d", r, p1 - p0, b->kv_len[r], need);
      for (int p = p0; p < p1; ++p) {
        if (b->page_ids[p] < 0 || b->page_ids[p] >= c->p.n_kv_pages)
          return fail(c, PIE_ERANGE, "request %d: page id %d outside [0, %d)", r, b->page_ids[p], c->p.n_kv_pages);
        for (int f = 0; f < F; ++f) blk_ids.push_back(b->page_ids[p] * F + f);
      }
      blk_indptr[r + 1] = (int32_t)blk_ids.size();
    }
    in_blocks = *b;
    in_blocks.page_indptr = blk_indptr.data();
    in_blocks.page_ids = blk_ids.data();
    b = &in_blocks;
  }
  std::vector<int32_t> tok_adapter;  // host only: adapter of each token's request
  std::vector<int32_t> used_adapters, lora_rows, lora_tile_ad;
  if (b->adapter_ids) {
    bool any = false;
    for (int r = 0; r < R; ++r) {
      const int ad = b->adapter_ids[r];
      if (ad < -1 || ad >= c->p.max_adapters)
        return fail(c, PIE_ERANGE, "request %d: adapter %d outside [-1, %d)", r, ad, c->p.max_adapters);
      any = any || ad >= 0;
    }
    if (any) tok_adapter.assign(T, -1);  // filled once the token ranges have been checked
  }
  std::vector<ReqInfo> reqs(R);
  std::vector<int32_t> tok_page(T), tok_slot(T), visit_phys, visit_logical, visit_pairs, dec_reqs;
  std::vector<int32_t> pos_from_embeds;  // positions recorded by embed_txt, when the batch names none
  if (!b->positions) pos_from_embeds.resize(T);
  std::vector<PrefillItem> pitems;
  const size_t n_mask_given = b->mask_indptr ? (size_t)b->mask_indptr[R] : 0;
  std::vector<uint32_t> extra_words;  // masks synthesised for requests that touch pages with token-level masks
  int rows_cap = 0;
  int64_t kv_bytes = 0, kv_bytes_dec = 0, flops = 0;
  const int64_t page_bytes = (int64_t)Hkv * 2 * PAGE * D * 2;
  for (int r = 0; r < R; ++r) {
    const int t0 = b->tok_indptr[r], t1 = b->tok_indptr[r + 1];
    const int n_new = t1 - t0, L = b->kv_len[r];
    const int p0 = b->page_indptr[r], p1 = b->page_indptr[r + 1];
    if (n_new <= 0) return fail(c, PIE_EINVAL, "request %d has no tokens", r);
    if (L < n_new) return fail(c, PIE_EINVAL, "request %d: kv_len %d < new tokens %d", r, L, n_new);
    const int n_pages = (L + PAGE - 1) / PAGE;
    if (p1 - p0 < n_pages) return fail(c, PIE_EINVAL, "request %d: %d pages listed, kv_len %d needs %d", r, p1 - p0, L, n_pages);
    for (int p = p0; p < p1; ++p)
      if (b->page_ids[p] < 0 || b->page_ids[p] >= n_pool_blocks)
        return fail(c, PIE_ERANGE, "request %d: page id %d outside [0, %d)", r, b->page_ids[p], n_pool_blocks);
    ReqInfo& q = reqs[r];
    q.tok0 = t0; q.n_new = n_new; q.kv_len = L;
    q.visit0 = (int32_t)visit_phys.size();
    q.wpr = 0; q.mask_off = 0; q.dec_index = -1; q.pair0 = 0;
    for (int i = 0; i < n_new; ++i) {
      const int t = t0 + i, j = L - n_new + i;
      if (b->in_embed_ids[t] < 0 || b->in_embed_ids[t] >= c->p.n_embeds)
        return fail(c, PIE_ERANGE, "token %d: input embed id %d outside [0, %d)", t, b->in_embed_ids[t], c->p.n_embeds);
      if (b->out_embed_ids[t] < -1 || b->out_embed_ids[t] >= c->p.n_embeds)
        return fail(c, PIE_ERANGE, "token %d: output embed id %d outside [-1, %d)", t, b->out_embed_ids[t], c->p.n_embeds);
      if (b->positions) {
        if (b->positions[t] < 0) return fail(c, PIE_ERANGE, "token %d: negative position", t);
      } else {
        pos_from_embeds[t] = c->embed_pos[b->in_embed_ids[t]];
        if (pos_from_embeds[t] < 0)
          return fail(c, PIE_EINVAL, "token %d: the batch names no positions and input embed %d carries none", t, b->in_embed_ids[t]);
      }
      tok_page[t] = b->page_ids[p0 + j / PAGE];
      tok_slot[t] = j % PAGE;
    }
    const bool has_mask = b->mask_indptr && b->mask_indptr[r + 1] > b->mask_indptr[r];
    const int wpr = (L + 31) / 32;
    if (has_mask && b->mask_indptr[r + 1] - b->mask_indptr[r] != (int64_t)wpr * n_new)
      return fail(c, PIE_EINVAL, "request %d: mask has %lld words, expected %lld", r,
                  (long long)(b->mask_indptr[r + 1] - b->mask_indptr[r]), (long long)wpr * n_new);
    // token-level page masks (mask_kvpage) in force on any page of the request: the request gets an explicit
    // mask of its own, the call's mask (given or causal) ANDed with the pages' bits
    bool page_masked = false;
    for (int pg = 0; pg < n_pages && !page_masked; ++pg) page_masked = c->page_mask[b->page_ids[p0 + pg]] != 0xFFFFu;
    const uint32_t* w = has_mask ? b->mask_words + b->mask_indptr[r] : nullptr;
    if (page_masked) {
      const size_t at = extra_words.size();
      extra_words.resize(at + (size_t)wpr * n_new);
      for (int k = 0; k < wpr; ++k) {
        uint32_t pm = c->page_mask[b->page_ids[p0 + 2 * k]];
        pm |= (2 * k + 1 < n_pages ? (uint32_t)c->page_mask[b->page_ids[p0 + 2 * k + 1]] : 0xFFFFu) << 16;
        for (int i = 0; i < n_new; ++i) {
          uint32_t base;
          if (has_mask) {
            base = w[(size_t)i * wpr + k];
          } else {  // causal on logical order: keys up to index lim
            const int lim = L - n_new + i, first = 32 * k;
            base = lim >= first + 31 ? 0xFFFFFFFFu : (lim < first ? 0u : (1u << (lim - first + 1)) - 1u);
          }
          extra_words[at + (size_t)i * wpr + k] = base & pm;
        }
      }
      q.wpr = wpr;
      q.mask_off = (int64_t)n_mask_given + (int64_t)at;
    } else if (has_mask) {
      q.wpr = wpr;
      q.mask_off = b->mask_indptr[r];
    }
    if (q.wpr > 0) {
      // a page is visited when any row has a visible key in it
      const uint32_t* we = page_masked ? extra_words.data() + (q.mask_off - (int64_t)n_mask_given) : w;
      std::vector<uint32_t> any(wpr, 0u);
      for (int i = 0; i < n_new; ++i)
        for (int k = 0; k < wpr; ++k) any[k] |= we[(size_t)i * wpr + k];
      for (int pg = 0; pg < n_pages; ++pg) {
        uint32_t bits = (any[pg >> 1] >> ((pg & 1) * 16)) & 0xFFFFu;
        int tail = L - pg * PAGE;
        if (tail < PAGE) bits &= (1u << tail) - 1u;
        if (bits) { visit_phys.push_back(b->page_ids[p0 + pg]); visit_logical.push_back(pg); }
      }
    } else {
      for (int pg = 0; pg < n_pages; ++pg) { visit_phys.push_back(b->page_ids[p0 + pg]); visit_logical.push_back(pg); }
    }
    q.n_visit = (int32_t)visit_phys.size() - q.visit0;
    const bool decode_path = n_new * G <= 16;  // query rows that fit the decode kernel's 16-column tile
    int64_t visited_pages = 0;
    if (decode_path) {
      q.dec_index = (int32_t)dec_reqs.size();
      dec_reqs.push_back(r);
      rows_cap = std::max(rows_cap, n_new * G);
      visited_pages = q.n_visit;
      kv_bytes_dec += visited_pages * page_bytes;
      flops += visited_pages * PAGE * (int64_t)n_new * c->m.n_q_heads * D * 4;
    } else {
      const int nqb = (n_new + 31) / 32;
      for (int qb = 0; qb < nqb; ++qb) pitems.push_back(PrefillItem{r, qb, 0, 0});
      q.pair0 = (int32_t)(visit_pairs.size() / 4);
      for (int v = 0; v < q.n_visit; v += 2) {
        const int v2 = v + 1 < q.n_visit ? v + 1 : v;
        visit_pairs.push_back(visit_phys[q.visit0 + v]);
        visit_pairs.push_back(visit_logical[q.visit0 + v]);
        visit_pairs.push_back(visit_phys[q.visit0 + v2]);
        visit_pairs.push_back(visit_logical[q.visit0 + v2]);
      }
      visited_pages = q.n_visit;  // each page is needed at least once
      if (q.wpr == 0) flops += (int64_t)c->m.n_q_heads * D * 4 * ((int64_t)n_new * (L - n_new) + (int64_t)n_new * (n_new + 1) / 2);
      else flops += visited_pages * PAGE * (int64_t)n_new * c->m.n_q_heads * D * 4;
    }
    kv_bytes += visited_pages * page_bytes;
  }
  if (!tok_adapter.empty())
    for (int r = 0; r < R; ++r) {
      const int ad = b->adapter_ids[r];
      for (int i = 0; i < reqs[r].n_new; ++i) tok_adapter[reqs[r].tok0 + i] = ad;
      if (ad >= 0 && std::find(used_adapters.begin(), used_adapters.end(), ad) == used_adapters.end()) used_adapters.push_back(ad);
    }
  // the adapted tokens grouped by adapter, each group padded to whole tiles of 32 rows
  for (int ad : used_adapters) {
    for (int t = 0; t < T; ++t)
      if (tok_adapter[t] == ad) lora_rows.push_back(t);
    while (lora_rows.size() % 32 != 0) lora_rows.push_back(-1);
    lora_tile_ad.resize(lora_rows.size() / 32, ad);
  }
  if (b->page_indptr[R] < 0) return fail(c, PIE_EINVAL, "bad page_indptr");
  if (validate) {
    std::unordered_set<int64_t> seen;
    seen.reserve((size_t)T * 2);
    for (int t = 0; t < T; ++t)
      if (!seen.insert((int64_t)tok_page[t] * PAGE + tok_slot[t]).second)
        return fail(c, PIE_ECONFLICT, "token %d writes (page %d, slot %d) that another token of the batch writes", t, tok_page[t], tok_slot[t]);
  }
  // Decode path.  Query columns are gathered into column groups of up to 16 columns that walk the same pages:
  // the rows of one request, or of several requests whose page tables name the same physical page at the same
  // logical index (shared prefixes), so that each K/V block is read once for all of them; what such requests
  // do not share stays in groups of their own.  The page pairs of all (column group, kv head) combinations form
  // one flat list that is cut into equal shares, one per wave, for as many waves as the chip keeps resident
  // (more when a share would exceed the 64 pairs whose page ids a wave holds in registers).  A share may cover
  // the end of one (group, head) and the start of the next; each such run is a segment with its own partial
  // result.  Every wave gets its page list (block index = page * Hkv + kv head, logical page) at a fixed
  // stride, two slots per pair.
  struct CGroup { std::vector<int> members; int rows; std::vector<int2> pages; };  // members: decode request indices
  std::vector<CGroup> cgroups;
  {
    std::unordered_map<int64_t, size_t> class_of;  // (rows, first physical page) -> index into classes
    std::vector<std::vector<int>> classes;
    for (size_t di = 0; di < dec_reqs.size(); ++di) {
      const int r = dec_reqs[di];
      const int rows = reqs[r].n_new * G;
      if (16 / rows < 2) {  // the request fills the 16 columns by itself
        classes.emplace_back(1, (int)di);
        continue;
      }
      const int64_t key = ((int64_t)rows << 32) | (uint32_t)b->page_ids[b->page_indptr[r]];
      auto ins = class_of.emplace(key, classes.size());
      if (ins.second) classes.emplace_back();
      classes[ins.first->second].push_back((int)di);
    }
    auto single = [&](int di, const std::vector<char>* skip) {
      const ReqInfo& q = reqs[dec_reqs[di]];
      CGroup g;
      g.members.push_back(di);
      g.rows = q.n_new * G;
      for (int v = 0; v < q.n_visit; ++v)
        if (!skip || !(*skip)[visit_logical[q.visit0 + v]])
          g.pages.push_back(make_int2(visit_phys[q.visit0 + v], visit_logical[q.visit0 + v]));
      if (!g.pages.empty() || !skip) cgroups.push_back(std::move(g));
    };
    for (const auto& cls : classes) {
      const int rows = reqs[dec_reqs[cls[0]]].n_new * G;
      const int cap = 16 / rows;
      for (size_t c0 = 0; c0 < cls.size(); c0 += cap) {
        const size_t c1 = std::min(cls.size(), c0 + cap);
        if (c1 - c0 < 2) { single(cls[c0], nullptr); continue; }
        // logical pages on which every member's table names the same physical page, visited by at least one
        int common = INT32_MAX;
        for (size_t k = c0; k < c1; ++k) common = std::min(common, (reqs[dec_reqs[cls[k]]].kv_len + PAGE - 1) / PAGE);
        std::vector<char> shared(common, 1), visited(common, 0);
        const int32_t* pg0 = b->page_ids + b->page_indptr[dec_reqs[cls[c0]]];
        for (size_t k = c0; k < c1; ++k) {
          const ReqInfo& q = reqs[dec_reqs[cls[k]]];
          const int32_t* pg = b->page_ids + b->page_indptr[dec_reqs[cls[k]]];
          for (int pgi = 0; pgi < common; ++pgi) if (pg[pgi] != pg0[pgi]) shared[pgi] = 0;
          for (int v = 0; v < q.n_visit; ++v)
            if (visit_logical[q.visit0 + v] < common) visited[visit_logical[q.visit0 + v]] = 1;
        }
        CGroup g;
        g.rows = rows;
        for (int pgi = 0; pgi < common; ++pgi) {
          shared[pgi] = shared[pgi] && visited[pgi];
          if (shared[pgi]) g.pages.push_back(make_int2(pg0[pgi], pgi));
        }
        if (g.pages.size() < 2) {  // nothing worth sharing
          for (size_t k = c0; k < c1; ++k) single(cls[k], nullptr);
          continue;
        }
        for (size_t k = c0; k < c1; ++k) g.members.push_back(cls[k]);
        cgroups.push_back(std::move(g));
        // what a member visits outside the shared pages (private suffix, pages beyond the shortest member)
        std::vector<char> skip;
        for (size_t k = c0; k < c1; ++k) {
          const int n_pg = (reqs[dec_reqs[cls[k]]].kv_len + PAGE - 1) / PAGE;
          skip.assign(n_pg, 0);
          std::copy(shared.begin(), shared.end(), skip.begin());
          single(cls[k], &skip);
        }
      }
    }
  }
  std::vector<DecodeCol> dcols(cgroups.size() * 16, DecodeCol{-1, 0, 0, 0, 0, 0, 0});
  std::vector<DecodeSeg> dsegs;
  std::vector<DecodeWave> dwaves;
  std::vector<int2> wave_pg;
  std::vector<std::vector<int32_t>> mref_lists(dec_reqs.size() * Hkv);
  int dslots = 2;
  int64_t kv_bytes_req = 0;  // bytes the decode kernel asks for after grouping
  {
    rows_cap = 1;
    int64_t total_pairs = 0;
    for (size_t gi = 0; gi < cgroups.size(); ++gi) {
      const CGroup& g = cgroups[gi];
      rows_cap = std::max(rows_cap, (int)g.members.size() * g.rows);
      total_pairs += (int64_t)((g.pages.size() + 1) / 2) * Hkv;
      kv_bytes_req += (int64_t)g.pages.size() * page_bytes;
      for (size_t mi = 0; mi < g.members.size(); ++mi) {
        const ReqInfo& q = reqs[dec_reqs[g.members[mi]]];
        for (int rr = 0; rr < g.rows; ++rr) {
          const int i_tok = rr / G;
          dcols[gi * 16 + mi * g.rows + rr] = DecodeCol{q.tok0 + i_tok, rr % G, q.kv_len, q.kv_len - q.n_new + i_tok,
                                                       q.wpr, 0, q.mask_off + (int64_t)i_tok * q.wpr};
        }
      }
    }
    // whole rounds of resident waves: when one round of 64-pair shares does not cover the list, the shares
    // shrink so that every round is full instead of leaving a nearly empty last one
    const int64_t rounds = std::max<int64_t>(1, (total_pairs + (int64_t)c->wave_slots * 64 - 1) / ((int64_t)c->wave_slots * 64));
    int64_t per_wave = (total_pairs + rounds * c->wave_slots - 1) / (rounds * c->wave_slots);
    per_wave = std::min<int64_t>(std::max<int64_t>(per_wave, 2), 64);
    dslots = (int)(2 * per_wave);
    wave_pg.reserve((size_t)((total_pairs + per_wave - 1) / per_wave + 1) * dslots);
    int filled = 0;
    DecodeWave cur{0, 0, 0, 0};
    auto close_wave = [&]() {
      cur.n_pairs = filled;
      dwaves.push_back(cur);
      wave_pg.resize(dwaves.size() * (size_t)dslots, make_int2(-1, 0));
      cur = DecodeWave{(int32_t)dsegs.size(), 0, 0, 0};
      filled = 0;
    };
    for (size_t gi = 0; gi < cgroups.size(); ++gi) {
      const CGroup& g = cgroups[gi];
      const int n_pg = (int)g.pages.size();
      const int P = (n_pg + 1) / 2;
      for (int hk = 0; hk < Hkv; ++hk) {
        int p = 0;
        while (p < P) {
          const int take = (int)std::min<int64_t>(per_wave - filled, P - p);
          for (size_t mi = 0; mi < g.members.size(); ++mi)  // partial rows start at segment * rows_cap (set below)
            mref_lists[(size_t)g.members[mi] * Hkv + hk].push_back((int32_t)(dsegs.size() * 16 + mi * g.rows));
          dsegs.push_back(DecodeSeg{(int32_t)gi, hk, take, 0});
          ++cur.n_seg;
          for (int pr = p; pr < p + take; ++pr)
            for (int e = 0; e < 2; ++e) {
              const int v = 2 * pr + e;
              wave_pg.push_back(v < n_pg ? make_int2(g.pages[v].x * Hkv + hk, g.pages[v].y) : make_int2(-1, 0));
            }
          p += take;
          filled += take;
          if (filled == per_wave) close_wave();
        }
      }
    }
    if (filled > 0) close_wave();
    // the kernel trusts this plan: check what it assumes before anything is launched from it
    const int64_t n_blocks = (int64_t)n_pool_blocks * Hkv;
    for (size_t w = 0; w < dwaves.size(); ++w) {
      const DecodeWave& dw = dwaves[w];
      int pairs = 0;
      bool ok = dw.n_seg > 0 && dw.seg0 >= 0 && dw.seg0 + dw.n_seg <= (int)dsegs.size();
      for (int sg = dw.seg0; ok && sg < dw.seg0 + dw.n_seg; ++sg) {
        pairs += dsegs[sg].n_pairs;
        ok = dsegs[sg].n_pairs > 0 && dsegs[sg].cgroup >= 0 && dsegs[sg].cgroup < (int)cgroups.size() &&
             dsegs[sg].hk >= 0 && dsegs[sg].hk < Hkv;
      }
      ok = ok && pairs == dw.n_pairs && dw.n_pairs > 0 && 2 * dw.n_pairs <= dslots;
      for (int j = 0; ok && j < 2 * dw.n_pairs; ++j) {
        const int2 e = wave_pg[w * dslots + j];
        ok = (e.x >= 0 || (j & 1)) && e.x < n_blocks && e.y >= 0;
      }
      if (!ok) return fail(c, PIE_EINVAL, "internal: inconsistent decode plan for wave %zu", w);
    }
    for (const DecodeCol& dc : dcols)
      if (dc.tok >= T || dc.hg < 0 || dc.hg >= G || (dc.tok >= 0 && dc.wpr > 0 && dc.mask_row + dc.wpr > (int64_t)(n_mask_given + extra_words.size())))
        return fail(c, PIE_EINVAL, "internal: inconsistent decode column");
  }
  // partial rows a (decode request, kv head) has to merge: segment * rows_cap + the request's first column
  std::vector<int32_t> mref_indptr(dec_reqs.size() * Hkv + 1, 0), mrefs;
  for (size_t i = 0; i < mref_lists.size(); ++i) {
    for (int32_t v : mref_lists[i]) mrefs.push_back((v / 16) * rows_cap + (v % 16));
    mref_indptr[i + 1] = (int32_t)mrefs.size();
  }
  // Prefill work list.  The hardware hands workgroup i to XCD i % 8, and every XCD has an L2 of its own: the
  // query blocks of one (request, kv head) read the same K/V pages, so they go to one XCD, next to each other in
  // its list (heavy blocks first), and that XCD's L2 serves all but the first read of a page.  The groups are
  // spread over the XCDs by cost, largest first onto the least loaded; while that leaves the XCDs uneven, groups
  // are cut into interleaved parts.  Requests whose page tables begin with the same physical page (a shared
  // prefix) form one family: the groups of a family for one kv head follow the family's first group onto its XCD
  // and sit next to each other there, so the shared K/V pages come from HBM once and from that L2 afterwards.
  // Lists are padded with empty slots to one length and interleaved.
  std::vector<int32_t> family(R);  // the first request whose visit list starts with the same physical block
  {
    std::unordered_map<int32_t, int32_t> first_with;
    for (int r = 0; r < R; ++r)
      family[r] = reqs[r].n_visit > 0 ? first_with.emplace(visit_phys[reqs[r].visit0], r).first->second : r;
  }
  auto pcost = [&](const PrefillItem& it) {
    const ReqInfo& q = reqs[it.r];
    return q.wpr ? (int64_t)q.n_visit * PAGE : (int64_t)(q.kv_len - q.n_new + std::min(q.n_new, it.qb * 32 + 32));
  };
  // Two launches: query blocks whose rows may see only a few keys (requests with a bitmap, and blocks of causal
  // requests that start within the first 64 keys) run with their softmax weights as bf16 pairs; all others with
  // plain bf16 weights.  Each launch gets a layout of its own.
  auto few_keys = [&](const PrefillItem& it) {
    const ReqInfo& q = reqs[it.r];
    return q.wpr > 0 || q.kv_len - q.n_new + it.qb * 32 < 64;
  };
  auto layout = [&](std::vector<PrefillItem> pitems) {
  std::stable_sort(pitems.begin(), pitems.end(), [&](const PrefillItem& x, const PrefillItem& y) {
    return x.r != y.r ? x.r < y.r : pcost(x) > pcost(y);
  });
  std::vector<PrefillItem> pwork;
  if (!pitems.empty()) {
    constexpr int N_XCD = 8;
    struct Unit { int32_t first, count, hk, part; int64_t cost; int32_t fam, order; };
    std::vector<int32_t> lists[N_XCD];
    for (int parts = 1;; parts *= 2) {
      std::vector<Unit> units;
      size_t i0 = 0;
      int32_t longest = 0;
      while (i0 < pitems.size()) {
        size_t i1 = i0;
        while (i1 < pitems.size() && pitems[i1].r == pitems[i0].r) ++i1;
        longest = std::max(longest, (int32_t)(i1 - i0));
        for (int hk = 0; hk < Hkv; ++hk)
          for (int pt = 0; pt < parts; ++pt) {
            int64_t cst = 0;
            for (size_t i = i0 + pt; i < i1; i += parts) cst += pcost(pitems[i]) + 64;
            if (cst > 0) units.push_back(Unit{(int32_t)i0, (int32_t)(i1 - i0), hk, pt, cst, family[pitems[i0].r], 0});
          }
        i0 = i1;
      }
      std::stable_sort(units.begin(), units.end(), [](const Unit& x, const Unit& y) { return x.cost > y.cost; });
      int64_t load[N_XCD] = {0}, total = 0;
      for (auto& l : lists) l.clear();
      std::vector<Unit> per_xcd[N_XCD];
      std::unordered_map<int64_t, std::pair<int, int>> home;  // (family, kv head, part) -> (XCD, rank on that XCD)
      for (Unit u : units) {
        const int64_t key = ((int64_t)u.fam * Hkv + u.hk) * parts + u.part;
        auto it = home.find(key);
        int best = 0;
        if (it != home.end()) {
          best = it->second.first;
          u.order = it->second.second;
        } else {
          for (int x = 1; x < N_XCD; ++x) if (load[x] < load[best]) best = x;
          u.order = (int)per_xcd[best].size();
          home.emplace(key, std::make_pair(best, u.order));
        }
        load[best] += u.cost; total += u.cost;
        per_xcd[best].push_back(u);
      }
      for (auto& v : per_xcd)  // a family's groups next to each other, families in the order their first group arrived
        std::stable_sort(v.begin(), v.end(), [](const Unit& x, const Unit& y) { return x.order < y.order; });
      const int64_t worst = *std::max_element(load, load + N_XCD);
      if (worst * N_XCD > total + total / 8 && parts < longest) continue;  // more than 1/8 over the mean: cut finer
      pwork.clear();
      size_t lmax = 0;
      std::vector<PrefillItem> flat[N_XCD];
      for (int x = 0; x < N_XCD; ++x) {
        for (const Unit& u : per_xcd[x])
          for (int32_t i = u.first + u.part; i < u.first + u.count; i += parts)
            flat[x].push_back(PrefillItem{pitems[i].r, pitems[i].qb, u.hk, 0});
        lmax = std::max(lmax, flat[x].size());
      }
      pwork.assign(lmax * N_XCD, PrefillItem{-1, 0, 0, 0});
      for (int x = 0; x < N_XCD; ++x)
        for (size_t i = 0; i < flat[x].size(); ++i) pwork[i * N_XCD + x] = flat[x][i];
      break;
    }
  }
  return pwork;
  };
  std::vector<PrefillItem> pitems_plain, pitems_pair;
  for (const PrefillItem& it : pitems) (few_keys(it) ? pitems_pair : pitems_plain).push_back(it);
  std::vector<PrefillItem> pwork = layout(std::move(pitems_plain));
  const size_t n_pwork_plain = pwork.size();
  {
    const std::vector<PrefillItem> lo = layout(std::move(pitems_pair));
    pwork.insert(pwork.end(), lo.begin(), lo.end());
  }

  pie_batch* pb = new pie_batch();
  pb->owner = c;
  pb->R = R; pb->T = T;
  pb->out_ids_host.assign(b->out_embed_ids, b->out_embed_ids + T);
  pb->n_dsegs = (int32_t)dsegs.size();
  pb->n_dwaves = (int32_t)dwaves.size();
  pb->dslots = dslots;
  pb->n_pitems = (int32_t)pitems.size();
  pb->n_pwork = (int32_t)n_pwork_plain;
  pb->n_pwork_lo = (int32_t)(pwork.size() - n_pwork_plain);
  pb->pwork_host = pwork;
  pb->n_dec_reqs = (int32_t)dec_reqs.size();
  pb->rows_cap = std::max(rows_cap, 1);
  pb->work[0] = kv_bytes; pb->work[1] = kv_bytes_dec; pb->work[2] = flops; pb->work[3] = (int64_t)visit_phys.size();
  {  // distinct pages the decode path visits: a stamp per pool page kept in the context (no clearing, no hashing)
    if (c->page_stamp.size() != (size_t)n_pool_blocks) c->page_stamp.assign(n_pool_blocks, 0u);
    if (++c->page_stamp_id == 0u) {  // wrapped: start over
      std::fill(c->page_stamp.begin(), c->page_stamp.end(), 0u);
      c->page_stamp_id = 1u;
    }
    const uint32_t id = c->page_stamp_id;
    int64_t distinct = 0;
    for (int r : dec_reqs)
      for (int v = reqs[r].visit0; v < reqs[r].visit0 + reqs[r].n_visit; ++v) {
        uint32_t& st = c->page_stamp[visit_phys[v]];  // page ids were range-checked when the visit list was built
        if (st != id) { st = id; ++distinct; }
      }
    pb->work[4] = distinct * page_bytes;
  }
  pb->work[5] = kv_bytes_req;
  Blob blob(c);
  const size_t o_in = blob.add(b->in_embed_ids, (size_t)T * 4), o_out = blob.add(b->out_embed_ids, (size_t)T * 4);
  const size_t o_pos = blob.add(b->positions ? b->positions : pos_from_embeds.data(), (size_t)T * 4), o_tp = blob.add(tok_page.data(), (size_t)T * 4);
  const size_t o_ts = blob.add(tok_slot.data(), (size_t)T * 4);
  const size_t o_lr = blob.add(lora_rows.empty() ? nullptr : lora_rows.data(), lora_rows.size() * 4, 4);
  const size_t o_lt = blob.add(lora_tile_ad.empty() ? nullptr : lora_tile_ad.data(), lora_tile_ad.size() * 4, 4);
  const size_t o_vp = blob.add(visit_phys.data(), visit_phys.size() * 4, 8);
  const size_t o_vl = blob.add(visit_logical.data(), visit_logical.size() * 4, 8);
  const size_t o_vq = blob.add(visit_pairs.data(), visit_pairs.size() * 4, 16);
  const size_t o_mw = blob.add(n_mask_given ? b->mask_words : nullptr, n_mask_given * 4, 0);
  if (!extra_words.empty()) {  // directly behind the caller's words: one array for the kernels
    blob.append(extra_words.data(), extra_words.size() * 4);
  }
  blob.append(nullptr, 4);
  const size_t o_rq = blob.add(reqs.data(), reqs.size() * sizeof(ReqInfo));
  const size_t o_di = blob.add(dsegs.data(), dsegs.size() * sizeof(DecodeSeg), 16);
  const size_t o_ws = blob.add(dwaves.data(), dwaves.size() * sizeof(DecodeWave), 16);
  const size_t o_wp = blob.add(wave_pg.data(), wave_pg.size() * sizeof(int2), 16);
  const size_t o_dc = blob.add(dcols.data(), dcols.size() * sizeof(DecodeCol), 16);
  const size_t o_mi = blob.add(mref_indptr.data(), mref_indptr.size() * 4, 4);
  const size_t o_mr = blob.add(mrefs.data(), mrefs.size() * 4, 4);
  const size_t o_pi = blob.add(pwork.data(), pwork.size() * sizeof(PrefillItem), 16);
  const size_t o_dr = blob.add(dec_reqs.data(), dec_reqs.size() * 4, 4);
  const size_t part_rows = (size_t)pb->n_dsegs * pb->rows_cap;
  const size_t o_po = blob.add(nullptr, 0, 0);  // metadata ends here; the partial buffers are device-only
  if (!blob.ok) {
    delete pb;
    return fail(c, PIE_ENOMEM, "pie_batch_create: no host memory for the batch image");
  }
  const size_t o_pm = (o_po + part_rows * D * 4 + 255) / 256 * 256;
  const size_t o_an = (o_pm + part_rows * 2 * 4 + 255) / 256 * 256;  // rotary angle table [T, D] floats
  const size_t total_bytes = o_an + (size_t)T * D * 4 + 256;
  if (c->host_only) {  // plan only: the work lists stay on the host and are dropped, the statistics remain
    pb->n_lora_tiles = (int)lora_tile_ad.size();
    pb->used_adapters = used_adapters;
    *out = pb;
    return PIE_OK;
  }
  hipError_t e = hipSuccess;
  {  // the smallest kept block that is large enough, else a new one (sizes in 1 MiB steps so that blocks get reused)
    int best = -1;
    for (int i = 0; i < (int)c->blob_pool.size(); ++i)
      if (c->blob_pool[i].second >= total_bytes && (best < 0 || c->blob_pool[i].second < c->blob_pool[best].second)) best = i;
    if (best >= 0) {
      pb->dev_blob = c->blob_pool[best].first;
      pb->dev_blob_bytes = c->blob_pool[best].second;
      c->blob_pool.erase(c->blob_pool.begin() + best);
    } else {
      pb->dev_blob_bytes = (total_bytes + (1u << 20) - 1) >> 20 << 20;
      e = hipMalloc(&pb->dev_blob, pb->dev_blob_bytes);
    }
  }
  if (e != hipSuccess) {
    delete pb;
    return fail(c, PIE_ENOMEM, "pie_batch_create: %s (%zu bytes)", hipGetErrorString(e), total_bytes);
  }
  // copy only the metadata part (everything before the partial buffers)
  e = hipMemcpyAsync(pb->dev_blob, blob.data(), blob.size, hipMemcpyHostToDevice, c->stream);
  if (e == hipSuccess)  // the rotary angles of the batch's positions: the same for every layer
    e = launch_rope_table(reinterpret_cast<const int32_t*>(reinterpret_cast<unsigned char*>(pb->dev_blob) + o_pos),
                          c->inv_freq, T, D, reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(pb->dev_blob) + o_an),
                          c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) {
    (void)hipFree(pb->dev_blob);
    delete pb;
    return fail(c, PIE_EHIP, "pie_batch_create: %s", hipGetErrorString(e));
  }
  unsigned char* d = reinterpret_cast<unsigned char*>(pb->dev_blob);
  pb->in_ids = (int32_t*)(d + o_in); pb->out_ids = (int32_t*)(d + o_out); pb->pos = (int32_t*)(d + o_pos);
  pb->tok_page = (int32_t*)(d + o_tp); pb->tok_slot = (int32_t*)(d + o_ts);
  pb->n_lora_tiles = (int)lora_tile_ad.size();
  pb->lora_rows = lora_rows.empty() ? nullptr : (int32_t*)(d + o_lr);
  pb->lora_tile_ad = lora_tile_ad.empty() ? nullptr : (int32_t*)(d + o_lt);
  pb->used_adapters = used_adapters;
  pb->visit_phys = (int32_t*)(d + o_vp); pb->visit_logical = (int32_t*)(d + o_vl); pb->visit_pairs = (int32_t*)(d + o_vq);
  pb->mask_words = (uint32_t*)(d + o_mw); pb->reqs = (ReqInfo*)(d + o_rq);
  pb->dsegs = (DecodeSeg*)(d + o_di); pb->dwaves = (DecodeWave*)(d + o_ws); pb->wave_pg = (int2*)(d + o_wp);
  pb->dcols = (DecodeCol*)(d + o_dc); pb->mref_indptr = (int32_t*)(d + o_mi); pb->mrefs = (int32_t*)(d + o_mr);
  pb->pitems = (PrefillItem*)(d + o_pi); pb->dec_reqs = (int32_t*)(d + o_dr);
  pb->part_o = (float*)(d + o_po); pb->part_ml = (float*)(d + o_pm);
  pb->rope_angles = (float*)(d + o_an);
  *out = pb;
  return PIE_OK;
}

extern "C" pie_status pie_batch_create(pie_ctx* c, const pie_forward_batch* b, int32_t validate, pie_batch** out) {
  return guarded(c, "pie_batch_create", [&]() { return pie_batch_create_impl(c, b, validate, out); });
}

extern "C" pie_status pie_batch_destroy(pie_ctx* c, pie_batch* b) {
  if (!b) return PIE_OK;
  if (c != b->owner) return fail(c, PIE_EINVAL, "pie_batch_destroy: the batch belongs to another context");
  if (c && !c->host_only) (void)hipStreamSynchronize(c->stream);  // no kernel may still read the batch
  if (b->dev_blob) {
    constexpr size_t POOL_BLOCKS = 8;
    if (c && c->blob_pool.size() < POOL_BLOCKS) c->blob_pool.emplace_back(b->dev_blob, b->dev_blob_bytes);
    else (void)hipFree(b->dev_blob);
  }
  delete b;
  return PIE_OK;
}

extern "C" pie_status pie_batch_plan_info(const pie_batch* b, int64_t* out) {
  if (!b || !out) return PIE_EINVAL;
  out[0] = b->n_dwaves;
  out[1] = b->n_dsegs;
  out[2] = b->dslots / 2;
  out[3] = b->n_pitems;
  out[4] = b->n_dec_reqs;
  out[5] = b->rows_cap;
  out[6] = b->n_pwork;
  out[7] = b->n_pwork_lo;
  return PIE_OK;
}

extern "C" pie_status pie_batch_prefill_work(const pie_batch* b, int32_t* out, int32_t cap, int32_t* n_entries) {
  if (!b || !n_entries || cap < 0 || (cap > 0 && !out)) return PIE_EINVAL;
  *n_entries = (int32_t)b->pwork_host.size();
  const int32_t n = std::min<int32_t>(cap, *n_entries);
  for (int32_t i = 0; i < n; ++i) {
    out[i * 3] = b->pwork_host[i].r;
    out[i * 3 + 1] = b->pwork_host[i].qb;
    out[i * 3 + 2] = b->pwork_host[i].hk;
  }
  return PIE_OK;
}

extern "C" pie_status pie_batch_work(const pie_batch* b, int64_t* out) {
  if (!b || !out) return PIE_EINVAL;
  for (int i = 0; i < 6; ++i) out[i] = b->work[i];
  return PIE_OK;
}

// ---------------------------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------------------------
namespace {
struct StageTimer {
  pie_ctx* c;
  StageTimer(pie_ctx* ctx, int first, int last) : c(ctx) {  // clears the stages this call owns
    if (c->timing) for (int i = first; i <= last; ++i) c->ev_used[i] = false;
  }
  void begin(int s) { if (c->timing) (void)hipEventRecord(c->ev[2 * s], c->stream); }
  void end(int s) { if (c->timing) { (void)hipEventRecord(c->ev[2 * s + 1], c->stream); c->ev_used[s] = true; } }
};
}  // namespace

// A batch can only run on the context that deserialised it (its device block, id ranges and launch plan belong to
// that context), and only when it has a device block at all (a planner's batch has none).
static pie_status check_batch(pie_ctx* c, const pie_batch* b, const char* who) {
  if (!b) return fail(c, PIE_EINVAL, "%s: null batch", who);
  if (b->owner != c) return fail(c, PIE_EINVAL, "%s: the batch was created by another context", who);
  if (!b->dev_blob) return fail(c, PIE_EINVAL, "%s: the batch has no device block (created by a planning context)", who);
  if (b->T > c->p.max_batch_tokens) return fail(c, PIE_EBATCH, "%s: batch larger than the context", who);
  return PIE_OK;
}

// One decoder layer.  x_in: wide [T, H] layer input, or null to read the batch's input Embeds; y_out: wide
// [T, H] destination of the layer output, or null to store it as bf16 into the batch's output Embeds.
// carry (optional): on entry, the number of split-K partial copies of the previous layer's down projection
// still waiting in the workspace (x_in = previous residual c->h + their sum has not been formed yet: the first
// norm does it); on return, the same for this layer's down projection (only when y_out is given).
static pie_status run_layer(pie_ctx* c, int32_t layer, const pie_batch* b, float* x_in, float* y_out, bool timed,
                            int* carry = nullptr) {
  const LayerWeights& L = c->layers[layer];
  const pie_model_desc& m = c->m;
  const int T = b->T, H = m.hidden, Hq = m.n_q_heads, Hkv = m.n_kv_heads, D = m.head_dim, I = m.mlp_dim;
  const int QKV = (Hq + 2 * Hkv) * D;
  hipStream_t s = c->stream;
  bf16_t* kv_layer = c->kv + (size_t)layer * c->kv_layer_elems;
  const bool was_timing = c->timing;
  if (!timed) c->timing = false;
  StageTimer tm(c, PIE_STAGE_NORM1, PIE_STAGE_DOWN);
  struct Restore { pie_ctx* c; bool v; ~Restore() { c->timing = v; } } restore{c, was_timing};
  EpiArgs e{};

  // LoRA pairs the batch's adapters carry in this layer, per projection
  bool lora[PIE_N_PROJ] = {false, false, false, false, false, false, false};
  if (b->n_lora_tiles > 0)
    for (int ad : b->used_adapters)
      for (int pj = 0; pj < PIE_N_PROJ; ++pj)
        if (c->lora[((size_t)ad * m.n_layers + layer) * PIE_N_PROJ + pj].rank > 0) lora[pj] = true;
  const int RM = round_up(c->p.max_lora_rank, 16), NL = m.n_layers, LT = b->n_lora_tiles;
  const bool lora_qkv = lora[PIE_PROJ_Q] || lora[PIE_PROJ_K] || lora[PIE_PROJ_V];
  // Small batches split their projections along K.  Where the next kernel reads the projection's output row by
  // row anyway, it sums the partial copies itself and the separate epilogue launch is saved: the rotary step
  // after QKV, the second norm after the output projection, the next layer's first norm after the down
  // projection.  An adapter update that sits between the two kernels rules this out.
  const int carried = (carry && x_in) ? *carry : 0;
  if (carry) *carry = 0;

  tm.begin(PIE_STAGE_NORM1);
  if (x_in && carried > 0)
    HIP_TRY(c, launch_splitk_resid_norm(c->splitk, carried, L.wdown.NB * 32, c->h, nullptr, nullptr, x_in, L.g1, c->xn, T, H, m.rms_eps, s));
  else if (x_in) HIP_TRY(c, launch_rmsnorm_f32(x_in, L.g1, c->xn, T, H, m.rms_eps, s));
  else HIP_TRY(c, launch_rmsnorm_embed(c->embeds, b->in_ids, L.g1, c->xn, T, H, m.rms_eps, s));
  tm.end(PIE_STAGE_NORM1);

  tm.begin(PIE_STAGE_QKV);
  int qkv_splits = 0;
  e = EpiArgs{EPI_STORE_BF16, c->qkv, QKV, nullptr, nullptr, nullptr, 0};
  HIP_TRY(c, launch_gemm(c->xn, H, T, L.wqkv, e, c->splitk, c->splitk_elems, c->wave_slots / 8, s,
                         lora_qkv ? nullptr : &qkv_splits));
  tm.end(PIE_STAGE_QKV);

  if (lora_qkv) {  // q, k, v share the normalised input
    const int KD = Hkv * D;
    const int ks = lora_ksplits(LT, 3, H, RM, c->lora_z_rows);
    HIP_TRY(c, launch_lora_down(c->xn, H, H, LT, 3, b->lora_rows, b->lora_tile_ad, c->lora_dev, layer, NL, PIE_PROJ_Q, c->lora_z, RM, ks, s));
    HIP_TRY(c, launch_lora_up(c->qkv, QKV, QKV, 3, Hq * D, KD, LT, b->lora_rows, b->lora_tile_ad, c->lora_dev, layer, NL, PIE_PROJ_Q, 0, c->lora_z, RM, ks, s));
  }

  tm.begin(PIE_STAGE_ROPE_APPEND);
  HIP_TRY(c, launch_rope_append(c->qkv, T, Hq, Hkv, D, b->pos, b->tok_page, b->tok_slot, b->rope_angles, kv_layer,
                                c->splitk, qkv_splits, L.wqkv.NB * 32, s));
  tm.end(PIE_STAGE_ROPE_APPEND);

  AttnArgs a{};
  a.q = c->qkv; a.q_stride = QKV; a.kv = kv_layer; a.out = c->attn; a.Hq = Hq; a.Hkv = Hkv; a.D = D;
  a.scale_log2 = (float)(1.4426950408889634 / std::sqrt((double)D));
  a.reqs = b->reqs; a.visit_phys = b->visit_phys; a.visit_logical = b->visit_logical; a.visit_pairs = b->visit_pairs; a.mask_words = b->mask_words;
  // Prefill attention first: it is bound by arithmetic, so the write-back of the lines the rotary step left dirty
  // (q rows and appended K/V of every prefill token) happens underneath it instead of slowing the decode kernel,
  // which is bound by HBM reads.
  if (b->n_pitems > 0) {
    tm.begin(PIE_STAGE_ATTN_PREFILL);
    HIP_TRY(c, launch_attn_prefill(a, b->pitems, b->n_pwork, false, s));
    HIP_TRY(c, launch_attn_prefill(a, b->pitems + b->n_pwork, b->n_pwork_lo, true, s));
    tm.end(PIE_STAGE_ATTN_PREFILL);
  }
  if (b->n_dec_reqs > 0) {
    tm.begin(PIE_STAGE_ATTN_DECODE);
    HIP_TRY(c, launch_attn_decode(a, b->dwaves, b->wave_pg, b->dslots, b->dsegs, b->dcols, b->n_dwaves, b->rows_cap, b->part_o, b->part_ml,
                                  /*read_once=*/b->work[5] <= b->work[4], s));
    tm.end(PIE_STAGE_ATTN_DECODE);
    tm.begin(PIE_STAGE_ATTN_MERGE);
    HIP_TRY(c, launch_attn_merge(a, b->dec_reqs, b->n_dec_reqs, b->mref_indptr, b->mrefs, b->rows_cap, b->part_o, b->part_ml, s));
    tm.end(PIE_STAGE_ATTN_MERGE);
  }

  tm.begin(PIE_STAGE_OPROJ);
  int o_splits = 0;
  e = EpiArgs{EPI_RESID_EMBED, c->h, H, c->embeds, b->in_ids, x_in, H};
  HIP_TRY(c, launch_gemm(c->attn, Hq * D, T, L.wo, e, c->splitk, c->splitk_elems, c->wave_slots / 8, s,
                         lora[PIE_PROJ_O] ? nullptr : &o_splits));
  tm.end(PIE_STAGE_OPROJ);

  if (lora[PIE_PROJ_O]) {  // h += scale * B (A attn), before the second norm reads h
    const int ks = lora_ksplits(LT, 1, Hq * D, RM, c->lora_z_rows);
    HIP_TRY(c, launch_lora_down(c->attn, Hq * D, Hq * D, LT, 1, b->lora_rows, b->lora_tile_ad, c->lora_dev, layer, NL, PIE_PROJ_O, c->lora_z, RM, ks, s));
    HIP_TRY(c, launch_lora_up(c->h, H, H, 1, 0, 0, LT, b->lora_rows, b->lora_tile_ad, c->lora_dev, layer, NL, PIE_PROJ_O, 0, c->lora_z, RM, ks, s));
  }

  tm.begin(PIE_STAGE_NORM2);
  if (o_splits > 0)
    HIP_TRY(c, launch_splitk_resid_norm(c->splitk, o_splits, L.wo.NB * 32, x_in, c->embeds, b->in_ids, c->h, L.g2, c->xn, T, H, m.rms_eps, s));
  else HIP_TRY(c, launch_rmsnorm_f32(c->h, L.g2, c->xn, T, H, m.rms_eps, s));
  tm.end(PIE_STAGE_NORM2);

  tm.begin(PIE_STAGE_GATEUP);
  if (lora[PIE_PROJ_GATE] || lora[PIE_PROJ_UP]) {
    // the update sits inside the nonlinearity: fp32 gate/up sums, update, then the SwiGLU product
    e = EpiArgs{EPI_STORE_F32, c->gu32, 2 * I, nullptr, nullptr, nullptr, 0};
    HIP_TRY(c, launch_gemm(c->xn, H, T, L.wgu, e, c->splitk, c->splitk_elems, c->wave_slots / 8, s));
    const int ks = lora_ksplits(LT, 2, H, RM, c->lora_z_rows);
    HIP_TRY(c, launch_lora_down(c->xn, H, H, LT, 2, b->lora_rows, b->lora_tile_ad, c->lora_dev, layer, NL, PIE_PROJ_GATE, c->lora_z, RM, ks, s));
    HIP_TRY(c, launch_lora_up(c->gu32, 2 * I, I, 2, 0, 0, LT, b->lora_rows, b->lora_tile_ad, c->lora_dev, layer, NL, PIE_PROJ_GATE, 0, c->lora_z, RM, ks, s));
    HIP_TRY(c, launch_lora_up(c->gu32, 2 * I, I, 2, 32, 0, LT, b->lora_rows, b->lora_tile_ad, c->lora_dev, layer, NL, PIE_PROJ_UP, 1, c->lora_z, RM, ks, s));
    HIP_TRY(c, launch_swiglu_f32(c->gu32, I, c->act, T, s));
  } else {
    e = EpiArgs{EPI_SWIGLU, c->act, I, nullptr, nullptr, nullptr, 0};
    HIP_TRY(c, launch_gemm(c->xn, H, T, L.wgu, e, c->splitk, c->splitk_elems, c->wave_slots / 8, s));
  }
  tm.end(PIE_STAGE_GATEUP);

  if (lora[PIE_PROJ_DOWN]) {  // added to the residual the down projection's epilogue reads
    const int ks = lora_ksplits(LT, 1, I, RM, c->lora_z_rows);
    HIP_TRY(c, launch_lora_down(c->act, I, I, LT, 1, b->lora_rows, b->lora_tile_ad, c->lora_dev, layer, NL, PIE_PROJ_DOWN, c->lora_z, RM, ks, s));
    HIP_TRY(c, launch_lora_up(c->h, H, H, 1, 0, 0, LT, b->lora_rows, b->lora_tile_ad, c->lora_dev, layer, NL, PIE_PROJ_DOWN, 0, c->lora_z, RM, ks, s));
  }

  tm.begin(PIE_STAGE_DOWN);
  e = EpiArgs{EPI_RESID_OUT, y_out, y_out ? H : 0, c->embeds, b->out_ids, c->h, H};
  HIP_TRY(c, launch_gemm(c->act, I, T, L.wdown, e, c->splitk, c->splitk_elems, c->wave_slots / 8, s,
                         (carry && y_out) ? carry : nullptr));
  tm.end(PIE_STAGE_DOWN);
  c->last_T = T;
  return PIE_OK;
}

extern "C" pie_status pie_forward(pie_ctx* c, int32_t layer, const pie_batch* b) {
  if (!c) return PIE_EINVAL;
  if (c->host_only) return fail(c, PIE_EINVAL, "pie_forward: the context only plans batches (pie_create_planner)");
  if (pie_status st = check_batch(c, b, "pie_forward")) return st;
  if (layer < 0 || layer >= c->m.n_layers) return fail(c, PIE_ERANGE, "pie_forward: layer %d of %d", layer, c->m.n_layers);
  if (!c->layers[layer].loaded) return fail(c, PIE_EINVAL, "pie_forward: layer %d has no weights", layer);
  return run_layer(c, layer, b, nullptr, nullptr, true);
}

extern "C" pie_status pie_forward_all(pie_ctx* c, const pie_batch* b) {
  if (!c) return PIE_EINVAL;
  if (c->host_only) return fail(c, PIE_EINVAL, "pie_forward_all: the context only plans batches (pie_create_planner)");
  if (pie_status st = check_batch(c, b, "pie_forward_all")) return st;
  const int NL = c->m.n_layers;
  for (int l = 0; l < NL; ++l)
    if (!c->layers[l].loaded) return fail(c, PIE_EINVAL, "pie_forward_all: layer %d has no weights", l);
  int carry = 0;
  for (int l = 0; l < NL; ++l) {
    // the layer output stays wide between layers; only the last layer stores bf16 Embeds
    pie_status st = run_layer(c, l, b, l == 0 ? nullptr : c->x32, l == NL - 1 ? nullptr : c->x32, NL == 1, &carry);
    if (st != PIE_OK) return st;
  }
  return PIE_OK;
}

extern "C" pie_status pie_forward_host(pie_ctx* c, int32_t layer, const pie_forward_batch* batch, int32_t validate) {
  pie_batch* pb = nullptr;
  pie_status st = pie_batch_create(c, batch, validate, &pb);
  if (st != PIE_OK) return st;
  st = pie_forward(c, layer, pb);
  pie_status st2 = pie_synchronize(c);
  pie_batch_destroy(c, pb);
  return st != PIE_OK ? st : st2;
}

// ---------------------------------------------------------------------------------------------
// get_next_dist
// ---------------------------------------------------------------------------------------------
// Argument checks of get_next_dist, everything but the ids themselves.
static pie_status check_dist_args(pie_ctx* c, const void* ids, int32_t n, int32_t top_k, float temperature,
                                  const void* out_ids, const void* out_probs) {
  if (!ids || n <= 0) return fail(c, PIE_EINVAL, "get_next_dist: null ids or n <= 0");
  if (!(temperature > 0.f) || !std::isfinite(temperature)) return fail(c, PIE_EINVAL, "temperature must be positive and finite");
  if (!c->head_loaded) return fail(c, PIE_EINVAL, "get_next_dist: no LM head loaded");
  if (n > c->p.max_dist_rows) return fail(c, PIE_EBATCH, "%d rows exceed max_dist_rows %d", n, c->p.max_dist_rows);
  if (top_k <= 0 || top_k > c->p.max_top_k || top_k > c->m.vocab)
    return fail(c, PIE_ERANGE, "top_k %d outside [1, min(max_top_k %d, vocab %d)]", top_k, c->p.max_top_k, c->m.vocab);
  if (!out_ids || !out_probs) return fail(c, PIE_EINVAL, "get_next_dist: null output");
  return PIE_OK;
}

// The kernels of get_next_dist over ids already on the device, with every intermediate buffer named by the caller
// (the context's workspace, or the static scratch array).
struct DistBuffers {
  const int32_t* ids;  // [n] embed ids
  bf16_t* en;          // [n, H] normalised rows
  float* logits;       // [n, V]
  float* splitk;       // split-K partial sums of the LM head
  size_t splitk_elems;
  unsigned long long* cand;  // [n, chunks, k]
  float* stats;              // [n, chunks, 2]
};
static pie_status run_dist(pie_ctx* c, const DistBuffers& w, int32_t n, int32_t top_k, float temperature,
                           int32_t* out_ids, float* out_probs) {
  const int H = c->m.hidden, V = c->m.vocab;
  hipStream_t s = c->stream;
  StageTimer tm(c, PIE_STAGE_HEAD_NORM, PIE_STAGE_TOPK);
  tm.begin(PIE_STAGE_HEAD_NORM);
  if (c->g_final) {
    HIP_TRY(c, launch_rmsnorm_embed(c->embeds, w.ids, c->g_final, w.en, n, H, c->m.rms_eps, s));
  } else {
    HIP_TRY(c, launch_embed_copy(c->embeds, w.ids, n, H, w.en, 0, s));
  }
  tm.end(PIE_STAGE_HEAD_NORM);
  tm.begin(PIE_STAGE_LM_HEAD);
  EpiArgs e{EPI_STORE_F32, w.logits, V, nullptr, nullptr, nullptr, 0};
  HIP_TRY(c, launch_gemm(w.en, H, n, c->wlm, e, w.splitk, w.splitk_elems, c->wave_slots / 8, s));
  tm.end(PIE_STAGE_LM_HEAD);
  tm.begin(PIE_STAGE_TOPK);
  HIP_TRY(c, launch_topk(w.logits, n, V, top_k, 1.0f / temperature, out_ids, out_probs, w.cand, w.stats, s));
  tm.end(PIE_STAGE_TOPK);
  c->last_dist_n = n;
  c->last_logits = w.logits;
  return PIE_OK;
}

extern "C" pie_status pie_get_next_dist(pie_ctx* c, const int32_t* embed_ids, int32_t n, int32_t top_k,
                                        float temperature, int32_t* out_ids, float* out_probs) {
  if (!c) return PIE_EINVAL;
  if (c->host_only) return fail(c, PIE_EINVAL, "pie_get_next_dist: the context only plans batches (pie_create_planner)");
  pie_status chk = check_dist_args(c, embed_ids, n, top_k, temperature, out_ids, out_probs);
  if (chk != PIE_OK) return chk;
  for (int i = 0; i < n; ++i)
    if (embed_ids[i] < 0 || embed_ids[i] >= c->p.n_embeds) return fail(c, PIE_ERANGE, "embed id %d at %d outside [0, %d)", embed_ids[i], i, c->p.n_embeds);
  pie_status st = stage_ids(c, embed_ids, nullptr, n);
  if (st != PIE_OK) return st;
  const DistBuffers w{c->ids_dev, c->en, c->logits, c->splitk, c->splitk_elems, c->topk_cand, c->topk_stats};
  return run_dist(c, w, n, top_k, temperature, out_ids, out_probs);
}

// Embed ids handed to the device as kernel arguments (no host-to-device copy, nothing to stage).
struct IdList { int32_t v[PIE_STATIC_DIST_ROWS]; };
__global__ void ids_from_args_kernel(IdList ids, int n, int32_t* __restrict__ dst) {
  const int i = threadIdx.x;
  if (i < n) dst[i] = ids.v[i];
}

extern "C" pie_status pie_get_next_dist_static(pie_ctx* c, const int32_t* embed_ids, int32_t n, int32_t top_k,
                                               float temperature, int32_t* out_ids, float* out_probs) {
  if (!c) return PIE_EINVAL;
  if (c->host_only) return fail(c, PIE_EINVAL, "pie_get_next_dist_static: the context only plans batches (pie_create_planner)");
  if (!embed_ids || n <= 0) return fail(c, PIE_EINVAL, "get_next_dist: null ids or n <= 0");
  if (!(temperature > 0.f) || !std::isfinite(temperature)) return fail(c, PIE_EINVAL, "temperature must be positive and finite");
  if (!c->head_loaded) return fail(c, PIE_EINVAL, "get_next_dist: no LM head loaded");
  if (!out_ids || !out_probs) return fail(c, PIE_EINVAL, "get_next_dist: null output");
  if (n > PIE_STATIC_DIST_ROWS) return fail(c, PIE_EBATCH, "%d rows exceed the %d rows of the allocation-free call", n, PIE_STATIC_DIST_ROWS);
  if (top_k <= 0 || top_k > 1024 || top_k > c->m.vocab)
    return fail(c, PIE_ERANGE, "top_k %d outside [1, min(1024, vocab %d)]", top_k, c->m.vocab);
  if (!c->static_scratch) return fail(c, PIE_EHIP, "the static scratch array of device %d was not found at pie_create", c->device);
  IdList ids{};
  for (int i = 0; i < n; ++i) {
    if (embed_ids[i] < 0 || embed_ids[i] >= c->p.n_embeds) return fail(c, PIE_ERANGE, "embed id %d at %d outside [0, %d)", embed_ids[i], i, c->p.n_embeds);
    ids.v[i] = embed_ids[i];
  }
  // carve the array: ids | normalised rows | logits | candidates | chunk statistics | split-K partials (the rest)
  const size_t H = (size_t)c->m.hidden, V = (size_t)c->m.vocab;
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  const size_t o_ids = 0, o_en = up(o_ids + PIE_STATIC_DIST_ROWS * 4), o_lg = up(o_en + (size_t)n * H * 2);
  const size_t o_cd = up(o_lg + (size_t)n * V * 4), o_st = up(o_cd + (size_t)n * 16 * top_k * 8);
  const size_t o_sk = up(o_st + (size_t)n * 16 * 2 * 4);
  if (o_sk > PIE_STATIC_SCRATCH_BYTES)
    return fail(c, PIE_EBATCH, "%d rows x vocab %zu x top_k %d need %zu bytes of scratch, the static array holds %u", n, V,
                top_k, o_sk, (unsigned)PIE_STATIC_SCRATCH_BYTES);
  unsigned char* base = c->static_scratch;  // the device address of this GPU's array, never the symbol itself
  // Nothing in the array has to start at zero: every kernel below writes each element it or a later kernel reads
  // (all n rows of en, logits, candidates (short chunks pad theirs), statistics and the partial sums that are used).
  ids_from_args_kernel<<<dim3(1), dim3(64), 0, c->stream>>>(ids, n, reinterpret_cast<int32_t*>(base + o_ids));
  HIP_TRY(c, hipGetLastError());
  const DistBuffers w{reinterpret_cast<const int32_t*>(base + o_ids), reinterpret_cast<bf16_t*>(base + o_en),
                      reinterpret_cast<float*>(base + o_lg), reinterpret_cast<float*>(base + o_sk),
                      (PIE_STATIC_SCRATCH_BYTES - o_sk) / sizeof(float),
                      reinterpret_cast<unsigned long long*>(base + o_cd), reinterpret_cast<float*>(base + o_st)};
  return run_dist(c, w, n, top_k, temperature, out_ids, out_probs);
}

static pie_status pie_forward_dist_impl(pie_ctx* c, const pie_batch* b, const int32_t* rows, int32_t n, int32_t top_k,
                                       float temperature, int32_t* out_ids, float* out_probs) {
  if (!c) return PIE_EINVAL;
  if (c->host_only) return fail(c, PIE_EINVAL, "pie_forward_dist: the context only plans batches (pie_create_planner)");
  if (pie_status stb = check_batch(c, b, "pie_forward_dist")) return stb;
  // every argument is checked before anything is enqueued
  pie_status st = check_dist_args(c, rows, n, top_k, temperature, out_ids, out_probs);
  if (st != PIE_OK) return st;
  std::vector<int32_t> ids(n);
  for (int i = 0; i < n; ++i) {
    if (rows[i] < 0 || rows[i] >= b->T) return fail(c, PIE_ERANGE, "row %d at %d outside [0, %d)", rows[i], i, b->T);
    ids[i] = b->out_ids_host[rows[i]];
    if (ids[i] < 0) return fail(c, PIE_EINVAL, "row %d stores no output Embed to take a distribution from", rows[i]);
  }
  st = pie_forward_all(c, b);
  if (st != PIE_OK) return st;
  return pie_get_next_dist(c, ids.data(), n, top_k, temperature, out_ids, out_probs);
}

extern "C" pie_status pie_forward_dist(pie_ctx* c, const pie_batch* b, const int32_t* rows, int32_t n, int32_t top_k,
                                       float temperature, int32_t* out_ids, float* out_probs) {
  return guarded(c, "pie_forward_dist", [&]() { return pie_forward_dist_impl(c, b, rows, n, top_k, temperature, out_ids, out_probs); });
}

extern "C" pie_status pie_synchronize(pie_ctx* c) {
  if (!c) return PIE_EINVAL;
  if (c->host_only) return PIE_OK;
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return PIE_OK;
}

// ---------------------------------------------------------------------------------------------
// observation points
// ---------------------------------------------------------------------------------------------
extern "C" pie_status pie_read_tap(pie_ctx* c, int32_t which, void* dst, int64_t n_elements) {
  if (!c || !dst) return PIE_EINVAL;
  if (c->host_only) return fail(c, PIE_EINVAL, "pie_read_tap: the context only plans batches (pie_create_planner)");
  const pie_model_desc& m = c->m;
  const int T = c->last_T, QD = m.n_q_heads * m.head_dim, QKV = (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim;
  switch (which) {
    case PIE_TAP_Q:
      if (n_elements != (int64_t)T * QD) return fail(c, PIE_EINVAL, "tap Q holds %lld elements", (long long)T * QD);
      HIP_TRY(c, hipMemcpy2DAsync(dst, (size_t)QD * 2, c->qkv, (size_t)QKV * 2, (size_t)QD * 2, T, hipMemcpyDeviceToDevice, c->stream));
      break;
    case PIE_TAP_ATTN:
      if (n_elements != (int64_t)T * QD) return fail(c, PIE_EINVAL, "tap ATTN holds %lld elements", (long long)T * QD);
      HIP_TRY(c, hipMemcpyAsync(dst, c->attn, (size_t)T * QD * 2, hipMemcpyDeviceToDevice, c->stream));
      break;
    case PIE_TAP_RESID:
      if (n_elements != (int64_t)T * m.hidden) return fail(c, PIE_EINVAL, "tap RESID holds %lld elements", (long long)T * m.hidden);
      HIP_TRY(c, hipMemcpyAsync(dst, c->h, (size_t)T * m.hidden * 4, hipMemcpyDeviceToDevice, c->stream));
      break;
    case PIE_TAP_ACT:
      if (n_elements != (int64_t)T * m.mlp_dim) return fail(c, PIE_EINVAL, "tap ACT holds %lld elements", (long long)T * m.mlp_dim);
      HIP_TRY(c, hipMemcpyAsync(dst, c->act, (size_t)T * m.mlp_dim * 2, hipMemcpyDeviceToDevice, c->stream));
      break;
    case PIE_TAP_LOGITS:
      if (n_elements != (int64_t)c->last_dist_n * m.vocab) return fail(c, PIE_EINVAL, "tap LOGITS holds %lld elements", (long long)c->last_dist_n * m.vocab);
      HIP_TRY(c, hipMemcpyAsync(dst, c->last_logits ? c->last_logits : c->logits, (size_t)n_elements * 4, hipMemcpyDeviceToDevice, c->stream));
      break;
    default:
      return fail(c, PIE_EINVAL, "unknown tap %d", which);
  }
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  return PIE_OK;
}

extern "C" pie_status pie_set_stage_timing(pie_ctx* c, int32_t enabled) {
  if (!c) return PIE_EINVAL;
  c->timing = enabled != 0;
  for (int i = 0; i < PIE_N_STAGES; ++i) c->ev_used[i] = false;
  return PIE_OK;
}

extern "C" pie_status pie_stage_times(pie_ctx* c, float* ms_out) {
  if (!c || !ms_out) return PIE_EINVAL;
  if (c->host_only) return fail(c, PIE_EINVAL, "pie_stage_times: the context only plans batches (pie_create_planner)");
  HIP_TRY(c, hipStreamSynchronize(c->stream));
  for (int i = 0; i < PIE_N_STAGES; ++i) {
    ms_out[i] = 0.f;
    if (c->ev_used[i]) HIP_TRY(c, hipEventElapsedTime(&ms_out[i], c->ev[2 * i], c->ev[2 * i + 1]));
  }
  return PIE_OK;
}
