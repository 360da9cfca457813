// Memory-bound helper kernels: weight tiling, RMSNorm, rotary step + KV append into pages,
// Embed / KvPage pool copies.
#include "internal.h"

// ---------------------------------------------------------------------------------------------
// Weight tiling: up to three [rows_i, K] matrices stacked (or two interleaved in 32-row blocks)
// into the tiled layout described in common.h.  One thread moves one 16-byte piece.
// ---------------------------------------------------------------------------------------------
__global__ void pack_weight_kernel(const bf16_t* __restrict__ s0, int r0, const bf16_t* __restrict__ s1, int r1,
                                   const bf16_t* __restrict__ s2, int r2, int K, int interleave,
                                   bf16_t* __restrict__ dst, int NB) {
  const int KB = K / 16;
  int64_t piece = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // one per (nb, kb, lane)
  int64_t total = (int64_t)NB * KB * 64;
  if (piece >= total) return;
  int lane = (int)(piece & 63);
  int64_t tile = piece >> 6;
  int kb = (int)(tile % KB);
  int nb = (int)(tile / KB);
  int n = nb * 32 + (lane & 31);
  int k = kb * 16 + (lane >> 5) * 8;
  const bf16_t* src = nullptr;
  if (interleave) {  // block 2b <- s0 rows [32b, 32b+32), block 2b+1 <- s1 rows [32b, 32b+32)
    int row = (nb >> 1) * 32 + (lane & 31);
    if (row < r0) src = ((nb & 1) ? s1 : s0) + (int64_t)row * K + k;
  } else {
    if (n < r0) src = s0 + (int64_t)n * K + k;
    else if (n < r0 + r1) src = s1 + (int64_t)(n - r0) * K + k;
    else if (n < r0 + r1 + r2) src = s2 + (int64_t)(n - r0 - r1) * K + k;
  }
  u32x4 v = {0, 0, 0, 0};
  if (src) v = *reinterpret_cast<const u32x4*>(src);
  *reinterpret_cast<u32x4*>(dst + piece * 8) = v;
}

hipError_t launch_pack_weight(const bf16_t* s0, int r0, const bf16_t* s1, int r1, const bf16_t* s2, int r2, int K,
                              int interleave, bf16_t* dst, int NB, hipStream_t s) {
  int64_t total = (int64_t)NB * (K / 16) * 64;
  int64_t blocks = (total + 255) / 256;
  pack_weight_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(s0, r0, s1, r1, s2, r2, K, interleave, dst, NB);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// RMSNorm: one workgroup per row, values kept in registers between the two passes.
// ---------------------------------------------------------------------------------------------
// The row comes from an Embed (NORM_EMBED), from a wide fp32 row (NORM_F32), or is first formed as residual +
// split-K partial sums of the projection before it (NORM_PARTIAL: partials added in split order, then the
// residual, exactly as the stand-alone split-K epilogue does, and the wide row is stored as well).
enum { NORM_EMBED = 0, NORM_F32 = 1, NORM_PARTIAL = 2 };
struct NormPartial {
  const float* part;    // [splits][rows][NP]
  int splits, NP, rows;
  const float* resid;   // [rows, H] fp32, or null: the residual is Embed ids[row]
  float* wide;          // [rows, H] fp32 destination of residual + sum
};

template <int SRC>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const void* __restrict__ xin, const int32_t* __restrict__ ids,
                                                      const bf16_t* __restrict__ gain, bf16_t* __restrict__ out,
                                                      int H, float eps, NormPartial np) {
  __shared__ float red[4];
  const int row = blockIdx.x;
  const int tid = threadIdx.x;
  constexpr int MAXV = 8;  // 8 elements per thread per pass of 2048 columns
  float vals[4][MAXV];
  float ss = 0.f;
  const int npass = (H + 2047) / 2048;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    int c = p * 2048 + tid * 8;
    if (p < npass && c < H) {
      if (SRC == NORM_EMBED) {
        const bf16_t* x = reinterpret_cast<const bf16_t*>(xin) + (int64_t)ids[row] * H + c;
        Pack16 pk;
        pk.u = *reinterpret_cast<const u32x4*>(x);
#pragma unroll
        for (int e = 0; e < 8; ++e) vals[p][e] = bf16_bits_to_f32(pk.s[e]);
      } else if (SRC == NORM_PARTIAL) {
        f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
        const float* pp = np.part + (int64_t)row * np.NP + c;
        const int64_t stride = (int64_t)np.rows * np.NP;
        int k = 0;
        for (; k + 8 <= np.splits; k += 8) {  // eight splits requested together, added in order
          f32x4 va[8], vb[8];
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            va[u] = *reinterpret_cast<const f32x4*>(pp + (k + u) * stride);
            vb[u] = *reinterpret_cast<const f32x4*>(pp + (k + u) * stride + 4);
          }
#pragma unroll
          for (int u = 0; u < 8; ++u) { a += va[u]; b += vb[u]; }
        }
        for (; k < np.splits; ++k) {
          a += *reinterpret_cast<const f32x4*>(pp + k * stride);
          b += *reinterpret_cast<const f32x4*>(pp + k * stride + 4);
        }
        if (np.resid != nullptr) {
          a += *reinterpret_cast<const f32x4*>(np.resid + (int64_t)row * H + c);
          b += *reinterpret_cast<const f32x4*>(np.resid + (int64_t)row * H + c + 4);
        } else {
          Pack16 pk;
          pk.u = *reinterpret_cast<const u32x4*>(reinterpret_cast<const bf16_t*>(xin) + (int64_t)ids[row] * H + c);
#pragma unroll
          for (int e = 0; e < 4; ++e) { a[e] += bf16_bits_to_f32(pk.s[e]); b[e] += bf16_bits_to_f32(pk.s[4 + e]); }
        }
        *reinterpret_cast<f32x4*>(np.wide + (int64_t)row * H + c) = a;
        *reinterpret_cast<f32x4*>(np.wide + (int64_t)row * H + c + 4) = b;
#pragma unroll
        for (int e = 0; e < 4; ++e) { vals[p][e] = a[e]; vals[p][4 + e] = b[e]; }
      } else {
        const float* x = reinterpret_cast<const float*>(xin) + (int64_t)row * H + c;
        f32x4 a = *reinterpret_cast<const f32x4*>(x);
        f32x4 b = *reinterpret_cast<const f32x4*>(x + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { vals[p][e] = a[e]; vals[p][4 + e] = b[e]; }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += vals[p][e] * vals[p][e];
    }
  }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  float tot = red[0] + red[1] + red[2] + red[3];
  float rstd = 1.0f / sqrtf(tot / (float)H + eps);
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    int c = p * 2048 + tid * 8;
    if (p < npass && c < H) {
      Pack16 g, o;
      g.u = *reinterpret_cast<const u32x4*>(gain + c);
#pragma unroll
      for (int e = 0; e < 8; ++e) o.h[e] = f32_to_bf16(vals[p][e] * rstd * bf16_bits_to_f32(g.s[e]));
      *reinterpret_cast<u32x4*>(out + (int64_t)row * H + c) = o.u;
    }
  }
}

hipError_t launch_rmsnorm_embed(const bf16_t* embeds, const int32_t* ids, const bf16_t* gain, bf16_t* out, int rows,
                                int H, float eps, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  rmsnorm_kernel<NORM_EMBED><<<dim3(rows), dim3(256), 0, s>>>(embeds, ids, gain, out, H, eps, NormPartial{});
  return hipGetLastError();
}
hipError_t launch_rmsnorm_f32(const float* x, const bf16_t* gain, bf16_t* out, int rows, int H, float eps,
                              hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  rmsnorm_kernel<NORM_F32><<<dim3(rows), dim3(256), 0, s>>>(x, nullptr, gain, out, H, eps, NormPartial{});
  return hipGetLastError();
}
hipError_t launch_splitk_resid_norm(const float* part, int splits, int NP, const float* resid, const bf16_t* embeds,
                                    const int32_t* ids, float* wide, const bf16_t* gain, bf16_t* out, int rows, int H,
                                    float eps, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (splits <= 0 || NP < H || (resid == nullptr && (embeds == nullptr || ids == nullptr))) return hipErrorInvalidValue;
  rmsnorm_kernel<NORM_PARTIAL><<<dim3(rows), dim3(256), 0, s>>>(embeds, ids, gain, out, H, eps,
                                                              NormPartial{part, splits, NP, rows, resid, wide});
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Rotary step + KV append.  qkv is [T, (Hq + 2 Hkv) * D] bf16.  A rotary thread handles the 8 pairs
// (c*8 + e, D/2 + c*8 + e) of `hpt` consecutive query/key heads of one token, so the 8 angles
// pos * theta^(-2i/D), evaluated in double (positions reach tens of thousands), are computed once for all of
// them; a value thread copies 16 consecutive elements.  Rotated queries are written back in place; rotated
// keys and values go to the token's page slot.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rope_append_kernel(bf16_t* __restrict__ qkv, int T, int Hq, int Hkv, int D,
                                                          const int32_t* __restrict__ pos,
                                                          const int32_t* __restrict__ tok_page,
                                                          const int32_t* __restrict__ tok_slot,
                                                          const float* __restrict__ angles,
                                                          bf16_t* __restrict__ kv_layer, int hpt,
                                                          const float* __restrict__ part, int splits, int NP) {
  // Eight consecutive values of token t from column `col` of its qkv row: read as stored, or (splits > 0) summed
  // in split order from the partials of the QKV product and rounded to bf16 like the stored row would be.
  auto load8 = [&](int t, int col) -> Pack16 {
    Pack16 r;
    if (splits > 0) {
      f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
      const float* pp = part + (int64_t)t * NP + col;
      const int64_t stride = (int64_t)T * NP;
      int k = 0;
      for (; k + 4 <= splits; k += 4) {
        f32x4 va[4], vb[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          va[u] = *reinterpret_cast<const f32x4*>(pp + (k + u) * stride);
          vb[u] = *reinterpret_cast<const f32x4*>(pp + (k + u) * stride + 4);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) { a += va[u]; b += vb[u]; }
      }
      for (; k < splits; ++k) {
        a += *reinterpret_cast<const f32x4*>(pp + k * stride);
        b += *reinterpret_cast<const f32x4*>(pp + k * stride + 4);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) { r.h[e] = f32_to_bf16(a[e]); r.h[4 + e] = f32_to_bf16(b[e]); }
    } else {
      r.u = *reinterpret_cast<const u32x4*>(qkv + (int64_t)t * NP + col);
    }
    return r;
  };
  const int cpt = D / 16;  // work pieces per head
  const int heads = Hq + 2 * Hkv, rot = Hq + Hkv;
  const int groups = (rot + hpt - 1) / hpt;
  const int64_t n_rot = (int64_t)T * groups * cpt, n_val = (int64_t)T * Hkv * cpt;
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_rot + n_val) return;
  if (idx < n_rot) {
    const int c = (int)(idx % cpt);
    const int g = (int)((idx / cpt) % groups);
    const int t = (int)(idx / ((int64_t)cpt * groups));
    const int page = tok_page[t], slot = tok_slot[t];
    float fc[8], fs[8];  // cos and sin of the token's 8 angles of this piece, from the batch's table
    {
      const float* ang = angles + (int64_t)t * D + c * 8;
      const f32x4 c0 = *reinterpret_cast<const f32x4*>(ang), c1 = *reinterpret_cast<const f32x4*>(ang + 4);
      const f32x4 s0 = *reinterpret_cast<const f32x4*>(ang + D / 2), s1 = *reinterpret_cast<const f32x4*>(ang + D / 2 + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) { fc[e] = c0[e]; fc[4 + e] = c1[e]; fs[e] = s0[e]; fs[4 + e] = s1[e]; }
    }
    const int h1 = min(rot, (g + 1) * hpt);
    for (int h = g * hpt; h < h1; ++h) {
      bf16_t* row = qkv + (int64_t)t * heads * D + (int64_t)h * D;
      Pack16 olo, ohi;
      const Pack16 lo = load8(t, h * D + c * 8), hi = load8(t, h * D + D / 2 + c * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float a = bf16_bits_to_f32(lo.s[e]), b = bf16_bits_to_f32(hi.s[e]);
        olo.h[e] = f32_to_bf16(a * fc[e] - b * fs[e]);
        ohi.h[e] = f32_to_bf16(b * fc[e] + a * fs[e]);
      }
      if (h < Hq) {
        *reinterpret_cast<u32x4*>(row + c * 8) = olo.u;
        *reinterpret_cast<u32x4*>(row + D / 2 + c * 8) = ohi.u;
      } else {
        bf16_t* blk = kv_layer + ((int64_t)page * Hkv + (h - Hq)) * (2 * PAGE * D);
        *reinterpret_cast<u32x4*>(blk + k_elem_offset(slot, c * 8)) = olo.u;
        *reinterpret_cast<u32x4*>(blk + k_elem_offset(slot, D / 2 + c * 8)) = ohi.u;
      }
    }
  } else {
    idx -= n_rot;
    const int c = (int)(idx % cpt);
    const int hv = (int)((idx / cpt) % Hkv);
    const int t = (int)(idx / ((int64_t)cpt * Hkv));
    const int page = tok_page[t], slot = tok_slot[t];
    bf16_t* blk = kv_layer + ((int64_t)page * Hkv + hv) * (2 * PAGE * D);
    // The V part keeps the 8 tokens of slots 8k .. 8k+7 next to each other for every d.  When the batch fills such
    // an octet with consecutive tokens (prefill), the thread of its first token writes all eight at once, 16 bytes
    // per d, and the other seven have nothing to do; single tokens (decode) store their 2-byte values one by one.
    const int t0 = t - (slot & 7);
    bool octet = t0 >= 0 && t0 + 7 < T;
#pragma unroll
    for (int i = 0; i < 8; ++i) octet = octet && tok_page[t0 + i] == page && tok_slot[t0 + i] == (slot & ~7) + i;
    if (octet) {
      if (t != t0) return;
      Pack16 a[8], b[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        a[i] = load8(t0 + i, (rot + hv) * D + c * 16);
        b[i] = load8(t0 + i, (rot + hv) * D + c * 16 + 8);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        Pack16 oa, ob;
#pragma unroll
        for (int i = 0; i < 8; ++i) { oa.s[i] = a[i].s[e]; ob.s[i] = b[i].s[e]; }
        *reinterpret_cast<u32x4*>(blk + v_elem_offset(slot, c * 16 + e, D)) = oa.u;
        *reinterpret_cast<u32x4*>(blk + v_elem_offset(slot, c * 16 + 8 + e, D)) = ob.u;
      }
      return;
    }
    const Pack16 a = load8(t, (rot + hv) * D + c * 16), b = load8(t, (rot + hv) * D + c * 16 + 8);
    uint16_t* dst = reinterpret_cast<uint16_t*>(blk);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      dst[v_elem_offset(slot, c * 16 + e, D)] = a.s[e];
      dst[v_elem_offset(slot, c * 16 + 8 + e, D)] = b.s[e];
    }
  }
}

// cos and sin of every (token, frequency) of a batch: angles[t][0 .. D/2) = cos, [D/2 .. D) = sin of
// pos[t] * inv_freq[i], evaluated in double precision and rounded to float.  Positions do not change from layer to
// layer, so the table is made once per batch and every layer's rotary step reads it.
__global__ void rope_table_kernel(const int32_t* __restrict__ pos, const double* __restrict__ inv_freq, int T, int half,
                                  float* __restrict__ angles) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)T * half) return;
  const int t = (int)(idx / half), i = (int)(idx % half);
  double sn, cs;
  sincos((double)pos[t] * inv_freq[i], &sn, &cs);
  angles[(int64_t)t * 2 * half + i] = (float)cs;
  angles[(int64_t)t * 2 * half + half + i] = (float)sn;
}

hipError_t launch_rope_table(const int32_t* pos, const double* inv_freq, int T, int D, float* angles, hipStream_t s) {
  const int64_t total = (int64_t)T * (D / 2);
  if (total <= 0) return hipSuccess;
  rope_table_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s>>>(pos, inv_freq, T, D / 2, angles);
  return hipGetLastError();
}

hipError_t launch_rope_append(bf16_t* qkv, int T, int Hq, int Hkv, int D, const int32_t* pos, const int32_t* tok_page,
                              const int32_t* tok_slot, const float* angles, bf16_t* kv_layer, const float* part,
                              int splits, int NP, hipStream_t s) {
  if (splits > 0 && (part == nullptr || NP < (Hq + 2 * Hkv) * D)) return hipErrorInvalidValue;
  if (splits <= 0) NP = (Hq + 2 * Hkv) * D;  // row length of the stored qkv
  // few tokens: one head per thread keeps enough threads in flight; many tokens: a thread walks several heads
  // with the same 8 angles
  const int hpt = T >= 1024 ? 8 : 1;
  const int groups = (Hq + Hkv + hpt - 1) / hpt;
  int64_t total = (int64_t)T * (groups + Hkv) * (D / 16);
  if (total <= 0) return hipSuccess;
  rope_append_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s>>>(qkv, T, Hq, Hkv, D, pos, tok_page,
                                                                                   tok_slot, angles, kv_layer, hpt,
                                                                                   part, splits, NP);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Pool copies for seeding and inspection.
// ---------------------------------------------------------------------------------------------
__global__ void embed_copy_kernel(bf16_t* __restrict__ embeds, const int32_t* __restrict__ ids, int n, int H,
                                  bf16_t* __restrict__ buf, int to_pool) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // one 16-byte piece
  int per_row = H / 8;
  if (idx >= (int64_t)n * per_row) return;
  int r = (int)(idx / per_row), c = (int)(idx % per_row) * 8;
  bf16_t* p = embeds + (int64_t)ids[r] * H + c;
  bf16_t* b = buf + (int64_t)r * H + c;
  if (to_pool) *reinterpret_cast<u32x4*>(p) = *reinterpret_cast<const u32x4*>(b);
  else *reinterpret_cast<u32x4*>(b) = *reinterpret_cast<const u32x4*>(p);
}

// embed_txt: Embed ids[r] receives row tok[r] of the embedding table, 16 bytes per thread.
__global__ void embed_gather_kernel(bf16_t* __restrict__ embeds, const int32_t* __restrict__ ids,
                                    const int32_t* __restrict__ tok, int n, int H, const bf16_t* __restrict__ table) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int per_row = H / 8;
  if (idx >= (int64_t)n * per_row) return;
  int r = (int)(idx / per_row), c = (int)(idx % per_row) * 8;
  *reinterpret_cast<u32x4*>(embeds + (int64_t)ids[r] * H + c) =
      *reinterpret_cast<const u32x4*>(table + (int64_t)tok[r] * H + c);
}

hipError_t launch_embed_gather(bf16_t* embeds, const int32_t* ids, const int32_t* tok, int n, int H,
                               const bf16_t* table, hipStream_t s) {
  int64_t total = (int64_t)n * (H / 8);
  if (total <= 0) return hipSuccess;
  embed_gather_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s>>>(embeds, ids, tok, n, H, table);
  return hipGetLastError();
}

hipError_t launch_embed_copy(bf16_t* embeds, const int32_t* ids, int n, int H, bf16_t* buf, int to_pool,
                             hipStream_t s) {
  int64_t total = (int64_t)n * (H / 8);
  if (total <= 0) return hipSuccess;
  embed_copy_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s>>>(embeds, ids, n, H, buf, to_pool);
  return hipGetLastError();
}

__global__ void kv_copy_kernel(bf16_t* __restrict__ kv_layer, const int32_t* __restrict__ pages,
                               const int32_t* __restrict__ slots, int n, int Hkv, int D, bf16_t* __restrict__ k,
                               bf16_t* __restrict__ v, int to_pool) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // one (token, head, d) element
  int64_t total = (int64_t)n * Hkv * D;
  if (idx >= total) return;
  int d = (int)(idx % D);
  int h = (int)((idx / D) % Hkv);
  int i = (int)(idx / ((int64_t)D * Hkv));
  uint16_t* blk = reinterpret_cast<uint16_t*>(kv_layer + ((int64_t)pages[i] * Hkv + h) * (2 * PAGE * D));
  uint16_t* kk = reinterpret_cast<uint16_t*>(k);
  uint16_t* vv = reinterpret_cast<uint16_t*>(v);
  int ko = k_elem_offset(slots[i], d), vo = v_elem_offset(slots[i], d, D);
  if (to_pool) {
    blk[ko] = kk[idx];
    blk[vo] = vv[idx];
  } else {
    kk[idx] = blk[ko];
    vv[idx] = blk[vo];
  }
}

hipError_t launch_kv_copy(bf16_t* kv_layer, const int32_t* pages, const int32_t* slots, int n, int Hkv, int D,
                          bf16_t* k, bf16_t* v, int to_pool, hipStream_t s) {
  int64_t total = (int64_t)n * Hkv * D;
  if (total <= 0) return hipSuccess;
  kv_copy_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s>>>(kv_layer, pages, slots, n, Hkv, D, k, v,
                                                                               to_pool);
  return hipGetLastError();
}

// copy_kvpage: token k of the call moves from (src page, src slot) to (dst page, dst slot), K and V, in every
// layer's pool (grid.y = layer); one thread per (token, kv head, element).
__global__ void kv_token_copy_kernel(bf16_t* __restrict__ kv, size_t layer_elems, const int32_t* __restrict__ sp,
                                     const int32_t* __restrict__ ss, const int32_t* __restrict__ dp,
                                     const int32_t* __restrict__ ds, int n, int Hkv, int D) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)n * Hkv * D) return;
  const int d = (int)(idx % D);
  const int h = (int)((idx / D) % Hkv);
  const int i = (int)(idx / ((int64_t)D * Hkv));
  uint16_t* pool = reinterpret_cast<uint16_t*>(kv + (size_t)blockIdx.y * layer_elems);
  const uint16_t* src = pool + ((int64_t)sp[i] * Hkv + h) * (2 * PAGE * D);
  uint16_t* dst = pool + ((int64_t)dp[i] * Hkv + h) * (2 * PAGE * D);
  dst[k_elem_offset(ds[i], d)] = src[k_elem_offset(ss[i], d)];
  dst[v_elem_offset(ds[i], d, D)] = src[v_elem_offset(ss[i], d, D)];
}

hipError_t launch_kv_token_copy(bf16_t* kv, size_t layer_elems, int n_layers, const int32_t* src_pages,
                                const int32_t* src_slots, const int32_t* dst_pages, const int32_t* dst_slots, int n,
                                int Hkv, int D, hipStream_t s) {
  int64_t total = (int64_t)n * Hkv * D;
  if (total <= 0 || n_layers <= 0) return hipSuccess;
  kv_token_copy_kernel<<<dim3((unsigned)((total + 255) / 256), (unsigned)n_layers), dim3(256), 0, s>>>(
      kv, layer_elems, src_pages, src_slots, dst_pages, dst_slots, n, Hkv, D);
  return hipGetLastError();
}
