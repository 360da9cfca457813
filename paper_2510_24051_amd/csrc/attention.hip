// Paged masked grouped-query attention on bf16 MFMA (32x32x16), for KvPages of 16 tokens.
//
// Both kernels walk a request's "visit list" (the pages that hold at least one visible key, in
// logical order) two pages at a time.  For a page pair and one kv head, a wave computes
//     S^T[32 keys, 32 query rows] = K[32, D] * Q^T[D, 32]          (D/16 MFMAs)
//     online softmax over the key axis (per lane 16 keys, one cross-lane step)
//     O^T[D, 32 query rows]      += V^T[D, 16 keys] * P^T[16, 32]   per page (D/32 MFMAs each)
// The page layout (internal.h) makes every K and V operand one coalesced 16-byte load per lane,
// and the S^T accumulator registers, converted to bf16, are already the P^T operand.
//
//   attn_decode  : requests with few new tokens (n_new * group <= 32 query rows).  HBM-bound.  The visit list
//                  is cut into chunks (split-K); one wave per (chunk, kv head) streams its pages and writes an
//                  unnormalised partial (running max, sum, O) that attn_merge combines.
//   attn_prefill : one workgroup per (request, 32-token query block, kv head), one wave per query head of
//                  the group; causal requests stop at the block's last visible page.
#include "internal.h"

template <int D>
struct AttnFrag {
  static constexpr int KS = D / 16;  // MFMA steps of the QK^T contraction
  static constexpr int DB = D / 32;  // 32-row blocks of O^T
};

// Running softmax state of one lane: query row (lane % 32), keys of lane group (lane / 32).
template <int D>
struct AttnState {
  f32x16 o[D / 32];
  float m;  // running max of scaled scores (log2 domain), -inf before the first visible key
  float l;  // this lane's share of the running sum
};

template <int D>
__device__ __forceinline__ void attn_init(AttnState<D>& st) {
#pragma unroll
  for (int b = 0; b < D / 32; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v) st.o[b][v] = 0.f;
  st.m = -INFINITY;
  st.l = 0.f;
}

// Visible-key bits of this lane's 8 keys (g*8 .. g*8+7) in logical page `pl`.
__device__ __forceinline__ uint32_t key_bits(const ReqInfo& rq, const uint32_t* __restrict__ mask_words, int i_tok,
                                             int pl, int g, bool row_valid) {
  if (!row_valid) return 0u;
  const int j0 = pl * PAGE + g * 8;
  int cnt = rq.kv_len - j0;  // keys of this group that exist
  cnt = cnt < 0 ? 0 : (cnt > 8 ? 8 : cnt);
  uint32_t bits = (1u << cnt) - 1u;
  if (rq.wpr > 0) {
    uint32_t w = mask_words[rq.mask_off + (int64_t)i_tok * rq.wpr + (pl >> 1)];
    bits &= (w >> ((pl & 1) * 16 + g * 8)) & 0xFFu;
  } else {
    int lim = rq.kv_len - rq.n_new + i_tok - j0 + 1;  // causal on logical order
    lim = lim < 0 ? 0 : (lim > 8 ? 8 : lim);
    bits &= (1u << lim) - 1u;
  }
  return bits;
}

// One page pair.  kf: K operands (rows 0-15 page a, 16-31 page b); va/vb: V^T operands of each page.
template <int D>
__device__ __forceinline__ void attn_step(AttnState<D>& st, const bf16x8 (&kf)[D / 16], const bf16x8 (&qf)[D / 16],
                                          const bf16x8 (&va)[D / 32], const bf16x8 (&vb)[D / 32], uint32_t bits_a,
                                          uint32_t bits_b, float scale_log2) {
  f32x16 s;
#pragma unroll
  for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
  for (int k = 0; k < D / 16; ++k) s = mfma32(kf[k], qf[k], s);
  // register v < 8: key g*8 + v of page a; v >= 8: key g*8 + v - 8 of page b
  float mx = -INFINITY;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const bool on = ((v < 8 ? (bits_a >> v) : (bits_b >> (v - 8))) & 1u) != 0u;
    s[v] = on ? s[v] * scale_log2 : -INFINITY;
    mx = fmaxf(mx, s[v]);
  }
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(st.m, mx);
  const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
  const float alpha = exp2f(st.m - m_safe);  // 0 while nothing was visible before
  float lsum = 0.f;
  Pack16 pa, pb;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const float p = exp2f(s[v] - m_safe);  // masked keys: exp2(-inf) = 0
    lsum += p;
    if (v < 8) pa.h[v] = f32_to_bf16(p);
    else pb.h[v - 8] = f32_to_bf16(p);
  }
  st.l = st.l * alpha + lsum;
  st.m = m_new;
#pragma unroll
  for (int b = 0; b < D / 32; ++b) {
#pragma unroll
    for (int v = 0; v < 16; ++v) st.o[b][v] *= alpha;
    st.o[b] = mfma32(va[b], pa.h, st.o[b]);
    st.o[b] = mfma32(vb[b], pb.h, st.o[b]);
  }
}

template <int D>
__device__ __forceinline__ void load_kv(const bf16_t* __restrict__ kv, int Hkv, int hk, int page_a, int page_b,
                                        int lane, bf16x8 (&kf)[D / 16], bf16x8 (&va)[D / 32], bf16x8 (&vb)[D / 32]) {
  const int64_t blk = 2 * PAGE * D;
  const bf16_t* ba = kv + ((int64_t)page_a * Hkv + hk) * blk;
  const bf16_t* bb = kv + ((int64_t)page_b * Hkv + hk) * blk;
  const int m = lane & 31, g = lane >> 5;
  const bf16_t* kbase = (m < 16 ? ba : bb) + g * 128 + (m & 15) * 8;
#pragma unroll
  for (int k = 0; k < D / 16; ++k) kf[k] = *reinterpret_cast<const bf16x8*>(kbase + k * 256);
  const int voff = PAGE * D + g * 256 + m * 8;
#pragma unroll
  for (int b = 0; b < D / 32; ++b) {
    va[b] = *reinterpret_cast<const bf16x8*>(ba + voff + b * 512);
    vb[b] = *reinterpret_cast<const bf16x8*>(bb + voff + b * 512);
  }
}

template <int D>
__device__ __forceinline__ void load_q(const bf16_t* __restrict__ qrow, bool valid, int g, bf16x8 (&qf)[D / 16]) {
#pragma unroll
  for (int k = 0; k < D / 16; ++k) {
    Pack16 p;
    p.u = u32x4{0, 0, 0, 0};
    if (valid) p.u = *reinterpret_cast<const u32x4*>(qrow + k * 16 + g * 8);
    qf[k] = p.h;
  }
}

// ------------------------------------------------------------------------------------------------
// decode: split-K partials
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_decode_kernel(AttnArgs a, const DecodeItem* __restrict__ items,
                                                          int n_items, int rows_cap, float* __restrict__ part_o,
                                                          float* __restrict__ part_ml) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int item = blockIdx.x * 4 + wave;
  const int hk = blockIdx.y;
  if (item >= n_items) return;
  const DecodeItem it = items[item];
  const ReqInfo rq = a.reqs[it.r];
  const int G = a.Hq / a.Hkv;
  const int rows = rq.n_new * G;
  const int qcol = lane & 31, g = lane >> 5;
  const bool valid = qcol < rows;
  const int i_tok = valid ? qcol / G : 0;
  const int hg = valid ? qcol % G : 0;
  bf16x8 qf[D / 16];
  load_q<D>(a.q + (int64_t)(rq.tok0 + i_tok) * a.q_stride + (hk * G + hg) * D, valid, g, qf);
  AttnState<D> st;
  attn_init<D>(st);
  for (int v = it.v0; v < it.v1; v += 2) {
    const bool has_b = v + 1 < it.v1;
    const int pl_a = a.visit_logical[v], pp_a = a.visit_phys[v];
    const int pl_b = has_b ? a.visit_logical[v + 1] : pl_a;
    const int pp_b = has_b ? a.visit_phys[v + 1] : pp_a;
    bf16x8 kf[D / 16], va[D / 32], vb[D / 32];
    load_kv<D>(a.kv, a.Hkv, hk, pp_a, pp_b, lane, kf, va, vb);
    const uint32_t bits_a = key_bits(rq, a.mask_words, i_tok, pl_a, g, valid);
    const uint32_t bits_b = has_b ? key_bits(rq, a.mask_words, i_tok, pl_b, g, valid) : 0u;
    attn_step<D>(st, kf, qf, va, vb, bits_a, bits_b, a.scale_log2);
  }
  const float l_tot = st.l + __shfl_xor(st.l, 32);
  if (!valid) return;
  const int64_t prow = ((int64_t)item * a.Hkv + hk) * rows_cap + qcol;
  if (g == 0) {
    part_ml[prow * 2] = st.m;
    part_ml[prow * 2 + 1] = l_tot;
  }
  float* po = part_o + prow * D;
#pragma unroll
  for (int b = 0; b < D / 32; ++b)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      f32x4 o4 = {st.o[b][q4 * 4], st.o[b][q4 * 4 + 1], st.o[b][q4 * 4 + 2], st.o[b][q4 * 4 + 3]};
      *reinterpret_cast<f32x4*>(po + b * 32 + q4 * 8 + g * 4) = o4;
    }
}

// One workgroup per (decode-path request, kv head); thread d combines the request's chunks for every row.
template <int D>
__global__ void attn_merge_kernel(AttnArgs a, const int32_t* __restrict__ dec_reqs, int rows_cap,
                                  const float* __restrict__ part_o, const float* __restrict__ part_ml) {
  const ReqInfo rq = a.reqs[dec_reqs[blockIdx.x]];
  const int hk = blockIdx.y, d = threadIdx.x;
  const int G = a.Hq / a.Hkv;
  const int rows = rq.n_new * G;
  for (int row = 0; row < rows; ++row) {
    float M = -INFINITY;
    for (int c = 0; c < rq.n_items; ++c)
      M = fmaxf(M, part_ml[(((int64_t)(rq.item0 + c) * a.Hkv + hk) * rows_cap + row) * 2]);
    float num = 0.f, den = 0.f;
    if (M != -INFINITY) {
      for (int c = 0; c < rq.n_items; ++c) {
        const int64_t prow = ((int64_t)(rq.item0 + c) * a.Hkv + hk) * rows_cap + row;
        const float w = exp2f(part_ml[prow * 2] - M);
        den += w * part_ml[prow * 2 + 1];
        num += w * part_o[prow * D + d];
      }
    }
    const float o = den > 0.f ? num / den : 0.f;
    const int i_tok = row / G, hg = row % G;
    a.out[(int64_t)(rq.tok0 + i_tok) * a.Hq * D + (hk * G + hg) * D + d] = f32_to_bf16(o);
  }
}

// ------------------------------------------------------------------------------------------------
// prefill
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(512) void attn_prefill_kernel(AttnArgs a, const PrefillItem* __restrict__ items) {
  const int lane = threadIdx.x & 63, hg = threadIdx.x >> 6;  // one wave per query head of the group
  const PrefillItem it = items[blockIdx.x];
  const int hk = blockIdx.y;
  const ReqInfo rq = a.reqs[it.r];
  const int G = a.Hq / a.Hkv;
  const int qcol = lane & 31, g = lane >> 5;
  const int i_tok = it.qb * 32 + qcol;
  const bool valid = i_tok < rq.n_new;
  const int i_ld = valid ? i_tok : rq.n_new - 1;
  bf16x8 qf[D / 16];
  load_q<D>(a.q + (int64_t)(rq.tok0 + i_ld) * a.q_stride + (hk * G + hg) * D, valid, g, qf);
  AttnState<D> st;
  attn_init<D>(st);
  int v_end = rq.n_visit;
  if (rq.wpr == 0) {  // inferred causal: the visit list is pages 0.. in order; stop at the block's last visible key
    int i_last = it.qb * 32 + 31;
    i_last = i_last < rq.n_new ? i_last : rq.n_new - 1;
    const int pages = (rq.kv_len - rq.n_new + i_last) / PAGE + 1;
    v_end = pages < v_end ? pages : v_end;
  }
  for (int v = 0; v < v_end; v += 2) {
    const bool has_b = v + 1 < v_end;
    const int va_i = rq.visit0 + v;
    const int pl_a = a.visit_logical[va_i], pp_a = a.visit_phys[va_i];
    const int pl_b = has_b ? a.visit_logical[va_i + 1] : pl_a;
    const int pp_b = has_b ? a.visit_phys[va_i + 1] : pp_a;
    bf16x8 kf[D / 16], va[D / 32], vb[D / 32];
    load_kv<D>(a.kv, a.Hkv, hk, pp_a, pp_b, lane, kf, va, vb);
    const uint32_t bits_a = key_bits(rq, a.mask_words, i_ld, pl_a, g, valid);
    const uint32_t bits_b = has_b ? key_bits(rq, a.mask_words, i_ld, pl_b, g, valid) : 0u;
    attn_step<D>(st, kf, qf, va, vb, bits_a, bits_b, a.scale_log2);
  }
  const float l_tot = st.l + __shfl_xor(st.l, 32);
  if (!valid) return;
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  bf16_t* orow = a.out + (int64_t)(rq.tok0 + i_tok) * a.Hq * D + (hk * G + hg) * D;
#pragma unroll
  for (int b = 0; b < D / 32; ++b)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      bf16x4 o4;
#pragma unroll
      for (int e = 0; e < 4; ++e) o4[e] = f32_to_bf16(st.o[b][q4 * 4 + e] * inv);
      *reinterpret_cast<bf16x4*>(orow + b * 32 + q4 * 8 + g * 4) = o4;
    }
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
hipError_t launch_attn_decode(const AttnArgs& a, const DecodeItem* items, int n_items, int rows_cap, float* part_o,
                              float* part_ml, hipStream_t s) {
  if (n_items <= 0) return hipSuccess;
  dim3 grid((n_items + 3) / 4, a.Hkv), block(256);
  if (a.D == 128) attn_decode_kernel<128><<<grid, block, 0, s>>>(a, items, n_items, rows_cap, part_o, part_ml);
  else if (a.D == 64) attn_decode_kernel<64><<<grid, block, 0, s>>>(a, items, n_items, rows_cap, part_o, part_ml);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_attn_merge(const AttnArgs& a, const int32_t* dec_reqs, int n_dec_reqs, int rows_cap,
                             const float* part_o, const float* part_ml, hipStream_t s) {
  if (n_dec_reqs <= 0) return hipSuccess;
  dim3 grid(n_dec_reqs, a.Hkv), block(a.D);
  if (a.D == 128) attn_merge_kernel<128><<<grid, block, 0, s>>>(a, dec_reqs, rows_cap, part_o, part_ml);
  else if (a.D == 64) attn_merge_kernel<64><<<grid, block, 0, s>>>(a, dec_reqs, rows_cap, part_o, part_ml);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_attn_prefill(const AttnArgs& a, const PrefillItem* items, int n_items, hipStream_t s) {
  if (n_items <= 0) return hipSuccess;
  const int G = a.Hq / a.Hkv;
  dim3 grid(n_items, a.Hkv), block(64 * G);
  if (a.D == 128) attn_prefill_kernel<128><<<grid, block, 0, s>>>(a, items);
  else if (a.D == 64) attn_prefill_kernel<64><<<grid, block, 0, s>>>(a, items);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}
