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
//                  the group; K/V page blocks shared through a four-stage LDS ring filled by direct-to-LDS
//                  loads; causal requests stop at the block's last visible page.
#include <type_traits>

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
// The softmax is kept lean: masking is skipped when the whole wave sees every key of the pair, the score
// scale is folded into the exponent's fused multiply-add, and the accumulators are rescaled only when some
// lane's running maximum actually moved.
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
  const uint32_t bits = bits_a | (bits_b << 8);
  if (__builtin_amdgcn_ballot_w64(bits != 0xFFFFu) != 0ull) {
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = ((bits >> v) & 1u) ? s[v] : -INFINITY;
  }
  const float mx_lo = max3(max3(s[0], s[1], s[2]), max3(s[3], s[4], s[5]), max3(s[6], s[7], s[8]));
  const float mx_hi = max3(max3(s[9], s[10], s[11]), max3(s[12], s[13], s[14]), s[15]);
  float mx = max3(mx_lo, mx_hi, mx_hi);
  mx = max_xor32(mx) * scale_log2;  // scale > 0; -inf stays -inf
  const float m_new = fmaxf(st.m, mx);
  const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
  if (__builtin_amdgcn_ballot_w64(m_new > st.m) != 0ull) {
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_safe);  // 0 while nothing was visible before
    st.l *= alpha;
#pragma unroll
    for (int b = 0; b < D / 32; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) st.o[b][v] *= alpha;
    st.m = m_new;
  }
  Pack16 pa, pb, la, lb;  // every weight as a bf16 pair hi + lo (see attn_softmax)
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[v], scale_log2, -m_safe));  // masked keys: exp2(-inf) = 0
    const bf16_t hi = f32_to_bf16(p);
    const bf16_t lo = f32_to_bf16(p - bf16_to_f32(hi));
    if (v < 8) { pa.h[v] = hi; la.h[v] = lo; }
    else { pb.h[v - 8] = hi; lb.h[v - 8] = lo; }
  }
  st.l = sum_bf16x8(lb.h, sum_bf16x8(la.h, sum_bf16x8(pb.h, sum_bf16x8(pa.h, st.l))));
#pragma unroll
  for (int b = 0; b < D / 32; ++b) {
    st.o[b] = mfma32(va[b], pa.h, st.o[b]);
    st.o[b] = mfma32(vb[b], pb.h, st.o[b]);
    st.o[b] = mfma32(va[b], la.h, st.o[b]);
    st.o[b] = mfma32(vb[b], lb.h, st.o[b]);
  }
}

constexpr float RESCALE_SLACK = 8.0f;

// The three phases of attn_step as separate functions, for kernels that overlap the QK^T MFMAs of the next
// pair with the softmax arithmetic of the current one.
template <int D>
__device__ __forceinline__ f32x16 attn_qk(const bf16x8 (&kf)[D / 16], const bf16x8 (&qf)[D / 16]) {
  f32x16 s;
#pragma unroll
  for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
  for (int k = 0; k < D / 16; ++k) s = mfma32(kf[k], qf[k], s);
  return s;
}

// LO: the softmax weights enter the PV product as bf16 pairs hi + lo (lo = the rounding error of hi, itself rounded
// to bf16), i.e. with 16 significand bits instead of 8, at the price of a second PV product.  A bf16 weight is off
// by up to 2^-9 relative; over hundreds of visible keys that averages out far below the rounding step of the bf16
// attention output, but a row that sees a handful of keys has outputs of order one and the weights' rounding
// flips the output's last bit for one element in six, which the output projection then sums over all heads.  The
// callers use LO where rows can see few keys (bitmap masks; causal blocks within the first 64 keys).
template <int D, bool LO = false>
__device__ __forceinline__ void attn_softmax(AttnState<D>& st, f32x16 s, uint32_t bits_a, uint32_t bits_b,
                                             float scale_log2, bf16x8& pa_out, bf16x8& pb_out, bf16x8* la_out = nullptr,
                                             bf16x8* lb_out = nullptr) {
  const uint32_t bits = bits_a | (bits_b << 8);
  if (__builtin_amdgcn_ballot_w64(bits != 0xFFFFu) != 0ull) {
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = ((bits >> v) & 1u) ? s[v] : -INFINITY;
  }
  const float mx_lo = max3(max3(s[0], s[1], s[2]), max3(s[3], s[4], s[5]), max3(s[6], s[7], s[8]));
  const float mx_hi = max3(max3(s[9], s[10], s[11]), max3(s[12], s[13], s[14]), s[15]);
  float mx = max3(mx_lo, mx_hi, mx_hi);
  mx = max_xor32(mx) * scale_log2;
  // The reference point st.m of the exponentials only has to stay within RESCALE_SLACK (in log2 units) of the
  // running maximum: weights up to 2^RESCALE_SLACK are harmless in fp32 sums and keep their relative precision
  // in bf16, and the final division by the sum of the same weights cancels the reference.  So the accumulators
  // are rescaled only when some row's maximum has moved by more than the slack, which after the first pairs of a
  // row almost never happens.
  const float m_new = fmaxf(st.m, mx);
  if (__builtin_amdgcn_ballot_w64(m_new > st.m + RESCALE_SLACK) != 0ull) {  // -inf + slack = -inf: first visible key
    const float m_to = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_to);  // 0 while nothing was visible before
    st.l *= alpha;
#pragma unroll
    for (int b = 0; b < D / 32; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) st.o[b][v] *= alpha;
    st.m = m_new;
  }
  const float m_safe = (st.m == -INFINITY) ? 0.f : st.m;
  Pack16 pa, pb, la, lb;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[v], scale_log2, -m_safe));
    const bf16_t hi = f32_to_bf16(p);
    if (v < 8) pa.h[v] = hi;
    else pb.h[v - 8] = hi;
    if (LO) {
      const bf16_t lo = f32_to_bf16(p - bf16_to_f32(hi));
      if (v < 8) la.h[v] = lo;
      else lb.h[v - 8] = lo;
    }
  }
  st.l = sum_bf16x8(pb.h, sum_bf16x8(pa.h, st.l));  // the normaliser of the weights as rounded for the PV product
  pa_out = pa.h;
  pb_out = pb.h;
  if (LO) {
    st.l = sum_bf16x8(lb.h, sum_bf16x8(la.h, st.l));
    *la_out = la.h;
    *lb_out = lb.h;
  }
}

template <int D>
__device__ __forceinline__ void attn_pv(AttnState<D>& st, const bf16x8 (&va)[D / 32], const bf16x8 (&vb)[D / 32],
                                        bf16x8 pa, bf16x8 pb) {
#pragma unroll
  for (int b = 0; b < D / 32; ++b) {
    st.o[b] = mfma32(va[b], pa, st.o[b]);
    st.o[b] = mfma32(vb[b], pb, st.o[b]);
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
// 16x16x32 MFMA: A is 16x32 (lane l: row l % 16, contraction elements (l / 16) * 8 .. + 8), B is 32x16 (lane l:
// column l % 16, same contraction elements), C/D 16x16 (lane l: column l % 16, register i is row (l / 16) * 4 + i).
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// Visible-key bits of the 4 keys j0 .. j0+3 of a page (j0 = logical index of the first), from a preloaded
// mask word (bitmap requests) or from the causal rule (keys up to logical index `lim`).
__device__ __forceinline__ uint32_t key_bits4(int kv_len, int lim, bool has_bitmap, uint32_t word, int pl, int quad,
                                              bool row_valid) {
  if (!row_valid) return 0u;
  const int j0 = pl * PAGE + quad * 4;
  int cnt = kv_len - j0;
  cnt = cnt < 0 ? 0 : (cnt > 4 ? 4 : cnt);
  uint32_t bits = (1u << cnt) - 1u;
  if (has_bitmap) {
    bits &= (word >> ((pl & 1) * 16 + quad * 4)) & 0xFu;
  } else {
    int c = lim - j0 + 1;
    c = c < 0 ? 0 : (c > 4 ? 4 : c);
    bits &= (1u << c) - 1u;
  }
  return bits;
}

// Decode attention (requests with n_new * group <= 16 query rows), HBM-bound.
// Grid: one wave per equal share of the flattened (column group, kv head, page pair) list.  A column group is
// up to 16 query columns that walk the same pages: the rows of one request, or of several requests that share
// physical pages at the same logical index (each K/V block is then read once for all of them); every column
// carries its own length, causal limit and mask row.  A share may cover the end of one (group, head) and the
// start of the next; each such run is a segment, and the wave writes one unnormalised partial (running max,
// sum, O) per segment and column.
// Per page pair and kv head, on 16x16x32 MFMAs (16 query columns, so accumulators are half the size of the
// 32-wide prefill tile and two waves per SIMD fit with K and V double-buffered in registers):
//     S^T[16 keys, 16 q]  = K_page[16, D] Q^T[D, 16]          per page, D/32 MFMAs; a K operand is one
//                                                              contiguous 1 KiB load per (page, 32 dims)
//     O^T[D, 16 q]       += V^T[D, 32 keys] P^T[32, 16]       D/16 MFMAs over both pages at once
// MFMA row r of a K operand is key swap23(r), so lane group g4 = lane / 16 ends up with keys
// 4*sigma(g4) .. +3 of each page (sigma swaps the two bits of g4); P^T is then the lane's own S registers.
// The wave's whole page list (block index = page * Hkv + kv head, and logical page number) sits at an address
// that depends on the wave index alone and is held across the lanes of two registers, so the first K/V request
// goes out after a single dependent load, and the K/V stream runs on across segment boundaries: the next pair
// (16 KiB per wave) is always requested before the current one is computed.  Segment descriptors, queries and
// (for bitmap requests) the mask words of pairs requested before a boundary are loaded at the boundary.
// NT: the K/V blocks are loaded non-temporally (batches in which no page is read twice).
template <int D, bool NT>
__global__ __launch_bounds__(256, 2) void attn_decode_kernel(AttnArgs a, const DecodeWave* __restrict__ waves,
                                                             const int2* __restrict__ wave_pg, int slots,
                                                             const DecodeSeg* __restrict__ segs,
                                                             const DecodeCol* __restrict__ cols, int n_waves,
                                                             int rows_cap, float* __restrict__ part_o,
                                                             float* __restrict__ part_ml) {
  constexpr int KS = D / 32;  // K operands per page
  constexpr int DB = D / 16;  // 16-row blocks of O^T
  const int lane = threadIdx.x & 63;
  const int gw = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));
  if (gw >= n_waves) return;
  const int G = a.Hq / a.Hkv;
  const int qcol = lane & 15, g4 = lane >> 4;
  const int quad = ((g4 & 1) << 1) | (g4 >> 1);  // sigma(g4): this lane group's key quad within a page
  constexpr int64_t blk = 2 * PAGE * D;
  const int koff = lane * 8;                                                    // + s32 * 512 elements
  const int voff = PAGE * D + (quad >> 1) * 256 + qcol * 8 + (quad & 1) * 4;    // + (d / 32) * 512 + ((d / 16) & 1) * 128
  // the wave's page list: slot 2j and 2j+1 are pair j (second block index -1: the pair has one page)
  const int2* wp = wave_pg + (int64_t)gw * slots;
  int2 id_lo = wp[min(lane, slots - 1)];        // clamped loads: lanes past the list are never consulted
  int2 id_hi = wp[min(lane + 64, slots - 1)];
  const DecodeWave wv = waves[gw];
  const int n_pairs = __builtin_amdgcn_readfirstlane(wv.n_pairs);
  int cur_sg = __builtin_amdgcn_readfirstlane(wv.seg0) - 1;
  int seg_end = 0;  // wave-local index of the first pair after the current segment

  // per-segment state (the column's own values: lane l works for column l % 16)
  int c_kv_len = 0, c_lim = 0;
  bool valid = false, has_bitmap = false;
  const uint32_t* mrow = a.mask_words;
  bf16x8 qf[KS];
#pragma unroll
  for (int k = 0; k < KS; ++k) { Pack16 p; p.u = u32x4{0, 0, 0, 0}; qf[k] = p.h; }
  f32x4 o[DB];
#pragma unroll
  for (int b = 0; b < DB; ++b) o[b] = f32x4{0.f, 0.f, 0.f, 0.f};
  float st_m = -INFINITY, st_l = 0.f;

  // two register sets, used alternately; the set index is a compile-time constant so they stay in registers
  bf16x8 ka[2][KS], kb[2][KS];
  bf16x4 va[2][DB], vb[2][DB];
  int pl_a[2] = {0, 0}, pl_b[2] = {0, 0};
  uint32_t mw_a[2] = {0u, 0u}, mw_b[2] = {0u, 0u};
  bool has_b[2] = {false, false};

  auto load_mask = [&](auto set_c) {
    constexpr int S = decltype(set_c)::value;
    if (has_bitmap && valid) { mw_a[S] = mrow[pl_a[S] >> 1]; mw_b[S] = mrow[pl_b[S] >> 1]; }
  };
  // Exactly one batch of loads per call, also past the last pair (then every lane reads the first bytes of the
  // last pair's blocks: a few cache lines, never used): with the same number of loads in flight on every path into
  // the loop header the compiler keeps exact wait counts, and the batch requested ahead stays in flight while the
  // current one is consumed.  (With conditional batches it waited for all outstanding loads in every compute.)
  auto ldk = [](const bf16x8* p) { return NT ? load_nt(p) : *p; };
  auto ldv = [](const bf16x4* p) { return NT ? load_nt(p) : *p; };
  auto fetch = [&](auto set_c, int j_req) {  // j_req is wave-uniform
    constexpr int S = decltype(set_c)::value;
    const bool real = j_req < n_pairs;
    const int j = real ? j_req : n_pairs - 1;
    const int ko = real ? koff : 0, vo = real ? voff : PAGE * D;
    const int src = (2 * j) & 63;
    const bool low = 2 * j < 64;
    const int pp_a = __builtin_amdgcn_readlane(low ? id_lo.x : id_hi.x, src);
    pl_a[S] = __builtin_amdgcn_readlane(low ? id_lo.y : id_hi.y, src);
    int pp_b = __builtin_amdgcn_readlane(low ? id_lo.x : id_hi.x, src + 1);
    pl_b[S] = __builtin_amdgcn_readlane(low ? id_lo.y : id_hi.y, src + 1);
    has_b[S] = pp_b >= 0;
    if (!has_b[S]) { pp_b = pp_a; pl_b[S] = pl_a[S]; }
    if (j < seg_end) load_mask(set_c);  // the pair belongs to the current segment: its mask row is known
    const bf16_t* pa_ = a.kv + (int64_t)pp_a * blk;
    const bf16_t* pb_ = a.kv + (int64_t)pp_b * blk;
#pragma unroll
    for (int k = 0; k < KS; ++k) {
      ka[S][k] = ldk(reinterpret_cast<const bf16x8*>(pa_ + ko + k * 512));
      kb[S][k] = ldk(reinterpret_cast<const bf16x8*>(pb_ + ko + k * 512));
    }
#pragma unroll
    for (int b = 0; b < DB; ++b) {
      const int vob = vo + (b >> 1) * 512 + (b & 1) * 128;
      va[S][b] = ldv(reinterpret_cast<const bf16x4*>(pa_ + vob));
      vb[S][b] = ldv(reinterpret_cast<const bf16x4*>(pb_ + vob));
    }
  };
  auto end_segment = [&]() {
    const float l_tot = sum_xor32(sum_xor16(st_l));
    if (valid) {
      const int64_t prow = (int64_t)cur_sg * rows_cap + qcol;
      if (g4 == 0) {
        part_ml[prow * 2] = st_m;
        part_ml[prow * 2 + 1] = l_tot;
      }
      float* po = part_o + prow * D + g4 * 4;
#pragma unroll
      for (int b = 0; b < DB; ++b) *reinterpret_cast<f32x4*>(po + b * 16) = o[b];
    }
  };
  auto begin_segment = [&](int j) {
    ++cur_sg;
    const DecodeSeg it = segs[cur_sg];
    const DecodeCol col = cols[(int64_t)it.cgroup * 16 + qcol];
    valid = col.tok >= 0;
    has_bitmap = col.wpr > 0;
    c_kv_len = col.kv_len;
    c_lim = col.lim;
    mrow = a.mask_words + col.mask_row;
    const bf16_t* qrow = a.q + (int64_t)(valid ? col.tok : 0) * a.q_stride + (it.hk * G + col.hg) * D + g4 * 8;
#pragma unroll
    for (int k = 0; k < KS; ++k) {
      Pack16 p;
      p.u = u32x4{0, 0, 0, 0};
      if (valid) p.u = *reinterpret_cast<const u32x4*>(qrow + k * 32);
      qf[k] = p.h;
    }
#pragma unroll
    for (int b = 0; b < DB; ++b) o[b] = f32x4{0.f, 0.f, 0.f, 0.f};
    st_m = -INFINITY;
    st_l = 0.f;
    seg_end = j + it.n_pairs;
  };
  auto compute = [&](auto set_c, auto other_c, int j) {
    constexpr int S = decltype(set_c)::value;
    if (j == seg_end) {  // wave-uniform: pair j opens the next segment
      if (j > 0) end_segment();
      begin_segment(j);
      // mask words of the pairs that were requested before the boundary
      load_mask(set_c);
      if (j + 1 < seg_end && j + 1 < n_pairs) load_mask(other_c);
    }
    const uint32_t bits_a = key_bits4(c_kv_len, c_lim, has_bitmap, mw_a[S], pl_a[S], quad, valid);
    const uint32_t bits_b = has_b[S] ? key_bits4(c_kv_len, c_lim, has_bitmap, mw_b[S], pl_b[S], quad, valid) : 0u;
    f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < KS; ++k) {
      sa = mfma16(ka[S][k], qf[k], sa);
      sb = mfma16(kb[S][k], qf[k], sb);
    }
    float sv[8];
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      sv[e] = ((bits_a >> e) & 1u) ? sa[e] * a.scale_log2 : -INFINITY;
      sv[4 + e] = ((bits_b >> e) & 1u) ? sb[e] * a.scale_log2 : -INFINITY;
      mx = fmaxf(mx, fmaxf(sv[e], sv[4 + e]));
    }
    mx = max_xor32(max_xor16(mx));
    const float m_new = fmaxf(st_m, mx);
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(st_m - m_safe);
    // The weights enter the PV product as bf16 pairs hi + lo (see attn_softmax): decode rows under sparse masks or
    // with short contexts see few keys, and the matrix cores are idle most of the time in this kernel anyway.
    Pack16 pp, pl;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float p = __builtin_amdgcn_exp2f(sv[e] - m_safe);
      pp.h[e] = f32_to_bf16(p);
      pl.h[e] = f32_to_bf16(p - bf16_to_f32(pp.h[e]));
    }
    st_l = sum_bf16x8(pl.h, sum_bf16x8(pp.h, st_l * alpha));  // the normaliser of the weights as the PV product sees them
    st_m = m_new;
#pragma unroll
    for (int b = 0; b < DB; ++b) {
      bf16x8 vv;
#pragma unroll
      for (int e = 0; e < 4; ++e) { vv[e] = va[S][b][e]; vv[4 + e] = vb[S][b][e]; }
#pragma unroll
      for (int e = 0; e < 4; ++e) o[b][e] *= alpha;
      o[b] = mfma16(vv, pp.h, o[b]);
      o[b] = mfma16(vv, pl.h, o[b]);
    }
  };
  if (n_pairs <= 0) return;
  std::integral_constant<int, 0> set0;
  std::integral_constant<int, 1> set1;
  fetch(set0, 0);
  for (int j = 0; j < n_pairs; j += 2) {
    fetch(set1, j + 1);
    compute(set0, set1, j);
    if (j + 1 >= n_pairs) break;
    fetch(set0, j + 2);
    compute(set1, set0, j + 1);
  }
  end_segment();
}

// One wave per (decode-path request, kv head, query row): lanes first share the (max, sum) pairs of the row's
// partials (one per segment in which the request has a column), then each lane combines D/64 output elements
// over the partials with independent loads.
template <int D>
__global__ __launch_bounds__(64) void attn_merge_kernel(AttnArgs a, const int32_t* __restrict__ dec_reqs,
                                                        const int32_t* __restrict__ mref_indptr,
                                                        const int32_t* __restrict__ mrefs, int rows_cap,
                                                        const float* __restrict__ part_o,
                                                        const float* __restrict__ part_ml) {
  const ReqInfo rq = a.reqs[dec_reqs[blockIdx.x]];
  const int hk = blockIdx.y, row = blockIdx.z, lane = threadIdx.x;
  const int G = a.Hq / a.Hkv;
  if (row >= rq.n_new * G) return;
  const int ref0 = mref_indptr[blockIdx.x * a.Hkv + hk];
  const int count = mref_indptr[blockIdx.x * a.Hkv + hk + 1] - ref0;
  constexpr int E = D / 64;
  float num[E];
#pragma unroll
  for (int e = 0; e < E; ++e) num[e] = 0.f;
  float M = -INFINITY;
  for (int c = lane; c < count; c += 64) M = fmaxf(M, part_ml[(int64_t)(mrefs[ref0 + c] + row) * 2]);
  M = wave_max(M);
  float den = 0.f;
  if (M != -INFINITY) {
    for (int c0 = 0; c0 < count; c0 += 64) {
      const int c = c0 + lane;
      float w = 0.f;
      int64_t prow = 0;
      if (c < count) {
        prow = mrefs[ref0 + c] + row;
        w = __builtin_amdgcn_exp2f(part_ml[prow * 2] - M);
        den += w * part_ml[prow * 2 + 1];
      }
      const int cnt = min(64, count - c0);
      // eight partial rows per round: their loads are independent and go out together
      for (int j0 = 0; j0 < cnt; j0 += 8) {
        float wj[8], v[8][E];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int j = min(j0 + u, cnt - 1);
          wj[u] = j0 + u < cnt ? __shfl(w, j) : 0.f;
          const float* po = part_o + (int64_t)__shfl((int)prow, j) * D + lane * E;
#pragma unroll
          for (int e = 0; e < E; ++e) v[u][e] = po[e];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
          for (int e = 0; e < E; ++e) num[e] += wj[u] * v[u][e];
      }
    }
    den = wave_sum(den);
  }
  const float inv = den > 0.f ? 1.0f / den : 0.f;
  const int i_tok = row / G, hg = row % G;
  bf16_t* out = a.out + (int64_t)(rq.tok0 + i_tok) * a.Hq * D + (hk * G + hg) * D + lane * E;
#pragma unroll
  for (int e = 0; e < E; ++e) out[e] = f32_to_bf16(num[e] * inv);
}

// N consecutive 1 KiB pieces global -> LDS (16 bytes per lane each); the immediate offset of the instruction
// moves both addresses, so one address computation serves the run.
template <int N>
__device__ __forceinline__ void lds_copy_run(const char* src, char* dst) {
  static_assert(N >= 1 && N <= 4, "the immediate offset reaches 4 KiB");
  const auto g = (const __attribute__((address_space(1))) void*)src;
  const auto l = (__attribute__((address_space(3))) void*)dst;
  __builtin_amdgcn_global_load_lds(g, l, 16, 0, 0);
  if constexpr (N > 1) __builtin_amdgcn_global_load_lds(g, l, 16, 1024, 0);
  if constexpr (N > 2) __builtin_amdgcn_global_load_lds(g, l, 16, 2048, 0);
  if constexpr (N > 3) __builtin_amdgcn_global_load_lds(g, l, 16, 3072, 0);
}

// ------------------------------------------------------------------------------------------------
// prefill
// ------------------------------------------------------------------------------------------------
// Prefill attention: one workgroup per (request, 32-token query block, kv head), one wave per query head of
// the group (G waves).  The K/V blocks of a page pair (16 KiB at D = 128) are shared by the group's waves through
// LDS: they are copied global -> LDS with direct-to-LDS loads (each wave issues its share, 1 KiB per
// instruction; the page block is already in operand order) into a ring of four stages, so the copies of the
// next three pairs are in flight while a pair is computed.  Every step issues exactly one copy batch (past the
// end it re-reads the last pair into a stage nobody consumes), which keeps the wait-counter arithmetic
// uniform: a pair has landed when at most two younger batches are outstanding.  Page ids are read with one scalar
// 16-byte load per pair, one pair ahead; mask words are fetched with the copy, three steps ahead of their use.
// Workgroups are listed per XCD by the host (all query blocks of a (request, kv head) on one XCD, whose L2 then
// serves the re-reads of its K/V); the lists are padded with empty items.
// LO: the softmax weights as bf16 pairs (see attn_softmax); the host lists the items that need it separately.
template <int D, int G, bool LO>
__global__ __launch_bounds__(64 * G, 2) void attn_prefill_kernel(AttnArgs a, const PrefillItem* __restrict__ items) {
  constexpr int BLK = 2 * PAGE * D;            // elements of one (page, head) block: K part then V part
  constexpr int PIECES = BLK * 2 / 1024;       // 1 KiB copy instructions per page block
  constexpr int IPW = 2 * PIECES / G;          // copy instructions per wave per pair
  static_assert(IPW * G == 2 * PIECES && 2 * IPW <= 63, "group size must divide the copy instructions");
  __shared__ __align__(16) bf16_t st0[2 * BLK], st1[2 * BLK], st2[2 * BLK], st3[2 * BLK];
  const int lane = threadIdx.x & 63, hg = threadIdx.x >> 6;
  const PrefillItem it = items[blockIdx.x];
  if (it.r < 0) return;  // padding of the per-XCD lists (uniform over the workgroup)
  const int hk = it.hk;
  const ReqInfo rq = a.reqs[it.r];
  const int qcol = lane & 31, g = lane >> 5, m = lane & 31;
  const int i_tok = it.qb * 32 + qcol;
  const bool valid = i_tok < rq.n_new;
  const int i_ld = valid ? i_tok : rq.n_new - 1;
  // requests with a bitmap are always listed in the launch with pair weights (their rows may see few keys)
  const bool has_bitmap = LO && rq.wpr > 0;
  bf16x8 qf[D / 16];
  load_q<D>(a.q + (int64_t)(rq.tok0 + i_ld) * a.q_stride + (hk * G + hg) * D, valid, g, qf);
  AttnState<D> st;
  attn_init<D>(st);
  int v_end = rq.n_visit;
  if (!has_bitmap) {  // inferred causal: the visit list is pages 0.. in order; stop at the block's last visible key
    int i_last = it.qb * 32 + 31;
    i_last = i_last < rq.n_new ? i_last : rq.n_new - 1;
    const int pages = (rq.kv_len - rq.n_new + i_last) / PAGE + 1;
    v_end = pages < v_end ? pages : v_end;
  }
  const int n_pairs = (v_end + 1) / 2;
  if (n_pairs > 0) {
    // Page ids are workgroup-uniform: one 16-byte scalar load per pair (physical and logical id of both pages)
    // through the constant address space (scalar loads do not count as vector memory operations, so waiting for
    // them never drains the copies in flight), one pair ahead of the pair that is started.
    typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
    typedef const __attribute__((address_space(4))) i32x4* const_i32x4;
    const const_i32x4 vis = (const_i32x4)(a.visit_pairs) + rq.pair0;
    i32x4 nx = {0, 0, 0, 0};
    auto fetch_ids = [&](int pair) { nx = vis[pair < n_pairs ? pair : n_pairs - 1]; };
    // Copies: this wave's pieces of a pair are consecutive 1 KiB pieces of one page block (of both blocks when
    // the workgroup is a single wave).  The source is a scalar base (page block) plus a per-lane offset, the
    // pieces of a run differ only in the instruction's immediate offset, which applies to both addresses.
    const int hgu = __builtin_amdgcn_readfirstlane(hg);
    constexpr int RUN = IPW < 4 ? IPW : 4;
    static_assert(IPW % RUN == 0 && PIECES % RUN == 0, "runs of copy pieces must not straddle page blocks");
    const char* kv_hk = reinterpret_cast<const char*>(a.kv + (int64_t)hk * BLK);
    const int64_t page_stride_b = (int64_t)a.Hkv * BLK * 2;
    const uint32_t lane_off = lane * 16;
    const uint32_t* mrow = a.mask_words + rq.mask_off + (int64_t)i_ld * rq.wpr;
    struct Meta { int pl_a, pl_b; bool has_b, full; uint32_t mw_a, mw_b; };
    Meta m0{}, m1{}, m2{}, m3{};
    // Inferred-causal blocks of 32 real rows: the first n_full pairs lie entirely at or below the first row's
    // limit (pages are visited in logical order without gaps when there is no bitmap), so every row sees all of
    // their keys, which the whole workgroup knows without any per-lane arithmetic.
    const bool rows_full = !has_bitmap && it.qb * 32 + 31 < rq.n_new;
    const int first_lim = rq.kv_len - rq.n_new + it.qb * 32;
    const int n_full = rows_full ? min(v_end / 2, (first_lim + 1) / 32) : 0;
    auto start_pair = [&](bf16_t* stage, int pair, Meta& md) {
      const int pc = pair < n_pairs ? pair : n_pairs - 1;
      const int pp_a = nx[0], pp_b = nx[2];  // fetched by the previous call (pairs are started in order)
      md.pl_a = nx[1];
      md.pl_b = nx[3];
      md.has_b = pc * 2 + 1 < v_end;
      fetch_ids(pair + 1);
      md.full = pair < n_full;
      if (has_bitmap && valid) { md.mw_a = mrow[md.pl_a >> 1]; md.mw_b = mrow[md.pl_b >> 1]; }
#pragma unroll
      for (int run = 0; run < IPW / RUN; ++run) {
        const int j0 = hgu * IPW + run * RUN;  // workgroup-wide copy index: page j0 / PIECES, piece j0 % PIECES
        const int page = j0 >= PIECES ? pp_b : pp_a;
        const char* src = kv_hk + (int64_t)page * page_stride_b + (j0 % PIECES) * 1024;
        lds_copy_run<RUN>(src + lane_off, reinterpret_cast<char*>(stage) + j0 * 1024);
      }
    };
    const int koff = (m < 16 ? 0 : BLK) + g * 128 + (m & 15) * 8;
    const int voff = PAGE * D + g * 256 + m * 8;
    auto bits_of = [&](uint32_t word, int pl) -> uint32_t {
      if (!valid) return 0u;
      const int j0 = pl * PAGE + g * 8;
      int cnt = rq.kv_len - j0;
      cnt = cnt < 0 ? 0 : (cnt > 8 ? 8 : cnt);
      uint32_t bits = (1u << cnt) - 1u;
      if (has_bitmap) {
        bits &= (word >> ((pl & 1) * 16 + g * 8)) & 0xFFu;
      } else {
        int lim = rq.kv_len - rq.n_new + i_ld - j0 + 1;
        lim = lim < 0 ? 0 : (lim > 8 ? 8 : lim);
        bits &= (1u << lim) - 1u;
      }
      return bits;
    };
    // QK^T of a pair (K part of its stage) and the rest of the step (softmax, then PV with the V part)
    auto scores = [&](const bf16_t* stage) {
      bf16x8 kf[D / 16];
#pragma unroll
      for (int k = 0; k < D / 16; ++k) kf[k] = *reinterpret_cast<const bf16x8*>(stage + koff + k * 256);
      return attn_qk<D>(kf, qf);
    };
    auto finish = [&](const bf16_t* stage, const Meta& md, const f32x16& sc) {
      uint32_t bits_a = 0xFFu, bits_b = 0xFFu;
      if (!md.full) {
        bits_a = bits_of(md.mw_a, md.pl_a);
        bits_b = md.has_b ? bits_of(md.mw_b, md.pl_b) : 0u;
      }
      // the V operands are requested before the softmax arithmetic, which hides their LDS latency
      bf16x8 va[D / 32], vb[D / 32];
#pragma unroll
      for (int bb = 0; bb < D / 32; ++bb) {
        va[bb] = *reinterpret_cast<const bf16x8*>(stage + voff + bb * 512);
        vb[bb] = *reinterpret_cast<const bf16x8*>(stage + BLK + voff + bb * 512);
      }
      __builtin_amdgcn_sched_barrier(0);
      bf16x8 pa, pb, la, lb;
      attn_softmax<D, LO>(st, sc, bits_a, bits_b, a.scale_log2, pa, pb, &la, &lb);
      attn_pv<D>(st, va, vb, pa, pb);
      if (LO) attn_pv<D>(st, va, vb, la, lb);
    };
#define PIE_WAIT_VM(n) PIE_S_WAIT_VMCNT(n)
    // Step i: the scores of pair i+1 are issued to the matrix cores first, so they run under the softmax
    // arithmetic of pair i.  A stage is read in two consecutive steps (K, then V), the ring has four stages,
    // two pairs are in flight.
    fetch_ids(0);
    start_pair(st0, 0, m0);
    start_pair(st1, 1, m1);
    start_pair(st2, 2, m2);
    PIE_WAIT_VM(2 * IPW);
    wg_barrier();
    f32x16 s_cur = scores(st0), s_next = s_cur;
    // One step: wait for the pair the scores need, start the copy three pairs ahead, scores of the next pair,
    // softmax and PV of the current one.  The loop body is four ring revolutions: at the loop header the compiler
    // waits for every copy in flight before the first LDS read (it cannot tell across the back edge which copies
    // may alias it), which empties the pipeline once per iteration.
#define PIE_STEP(SA, MA, SCUR, SB, SNEXT, SC, MC, AHEAD)   \
    PIE_WAIT_VM(IPW);                                      \
    wg_barrier();                                          \
    start_pair(SC, p + (AHEAD), MC);                       \
    SNEXT = scores(SB);                                    \
    finish(SA, MA, SCUR);
#define PIE_REVOLUTION(BASE)                                         \
    PIE_STEP(st0, m0, s_cur, st1, s_next, st3, m3, (BASE) + 3)       \
    if (p + (BASE) + 1 >= n_pairs) break;                            \
    PIE_STEP(st1, m1, s_next, st2, s_cur, st0, m0, (BASE) + 4)       \
    if (p + (BASE) + 2 >= n_pairs) break;                            \
    PIE_STEP(st2, m2, s_cur, st3, s_next, st1, m1, (BASE) + 5)       \
    if (p + (BASE) + 3 >= n_pairs) break;                            \
    PIE_STEP(st3, m3, s_next, st0, s_cur, st2, m2, (BASE) + 6)
    for (int p = 0; p < n_pairs; p += 16) {
      PIE_REVOLUTION(0)
      if (p + 4 >= n_pairs) break;
      PIE_REVOLUTION(4)
      if (p + 8 >= n_pairs) break;
      PIE_REVOLUTION(8)
      if (p + 12 >= n_pairs) break;
      PIE_REVOLUTION(12)
    }
#undef PIE_REVOLUTION
#undef PIE_STEP
    PIE_WAIT_VM(0);
#undef PIE_WAIT_VM
  }
  const float l_tot = sum_xor32(st.l);
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

// Variant without LDS: every wave loads its own K/V operands from global memory (the group's waves meet in L1).
template <int D>
__global__ __launch_bounds__(512) void attn_prefill_direct_kernel(AttnArgs a, const PrefillItem* __restrict__ items) {
  const int lane = threadIdx.x & 63, hg = threadIdx.x >> 6;  // one wave per query head of the group
  const PrefillItem it = items[blockIdx.x];
  if (it.r < 0) return;  // padding of the per-XCD lists (uniform over the workgroup)
  const int hk = it.hk;
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
  const float l_tot = sum_xor32(st.l);
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
hipError_t launch_attn_decode(const AttnArgs& a, const DecodeWave* waves, const int2* wave_pg, int slots,
                              const DecodeSeg* segs, const DecodeCol* cols, int n_waves, int rows_cap, float* part_o,
                              float* part_ml, bool read_once, hipStream_t s) {
  if (n_waves <= 0) return hipSuccess;
  if (slots < 2 || slots > 128 || (slots & 1)) return hipErrorInvalidValue;  // the page list must fit two registers
  dim3 grid((n_waves + 3) / 4), block(256);
  // Requests that alias pages (shared prefixes) read them again and again out of the caches; everything else is
  // read once and streams past them.
  if (a.D == 128 && read_once)
    attn_decode_kernel<128, true><<<grid, block, 0, s>>>(a, waves, wave_pg, slots, segs, cols, n_waves, rows_cap, part_o, part_ml);
  else if (a.D == 128)
    attn_decode_kernel<128, false><<<grid, block, 0, s>>>(a, waves, wave_pg, slots, segs, cols, n_waves, rows_cap, part_o, part_ml);
  else if (a.D == 64 && read_once)
    attn_decode_kernel<64, true><<<grid, block, 0, s>>>(a, waves, wave_pg, slots, segs, cols, n_waves, rows_cap, part_o, part_ml);
  else if (a.D == 64)
    attn_decode_kernel<64, false><<<grid, block, 0, s>>>(a, waves, wave_pg, slots, segs, cols, n_waves, rows_cap, part_o, part_ml);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_attn_merge(const AttnArgs& a, const int32_t* dec_reqs, int n_dec_reqs, const int32_t* mref_indptr,
                             const int32_t* mrefs, int rows_cap, const float* part_o, const float* part_ml,
                             hipStream_t s) {
  if (n_dec_reqs <= 0) return hipSuccess;
  dim3 grid(n_dec_reqs, a.Hkv, rows_cap), block(64);
  if (a.D == 128) attn_merge_kernel<128><<<grid, block, 0, s>>>(a, dec_reqs, mref_indptr, mrefs, rows_cap, part_o, part_ml);
  else if (a.D == 64) attn_merge_kernel<64><<<grid, block, 0, s>>>(a, dec_reqs, mref_indptr, mrefs, rows_cap, part_o, part_ml);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

template <int D, bool LO>
static hipError_t launch_prefill_d(const AttnArgs& a, const PrefillItem* items, int n_items, hipStream_t s) {
  const int G = a.Hq / a.Hkv;
  dim3 grid(n_items), block(64 * G);
  if (G == 1) attn_prefill_kernel<D, 1, LO><<<grid, block, 0, s>>>(a, items);
  else if (G == 2) attn_prefill_kernel<D, 2, LO><<<grid, block, 0, s>>>(a, items);
  else if (G == 4) attn_prefill_kernel<D, 4, LO><<<grid, block, 0, s>>>(a, items);
  else if (G == 8) attn_prefill_kernel<D, 8, LO><<<grid, block, 0, s>>>(a, items);
  else attn_prefill_direct_kernel<D><<<grid, block, 0, s>>>(a, items);  // other group sizes: no LDS sharing
  return hipGetLastError();
}

hipError_t launch_attn_prefill(const AttnArgs& a, const PrefillItem* items, int n_items, bool pair_weights,
                               hipStream_t s) {
  if (n_items <= 0) return hipSuccess;
  if (a.D == 128)
    return pair_weights ? launch_prefill_d<128, true>(a, items, n_items, s) : launch_prefill_d<128, false>(a, items, n_items, s);
  if (a.D == 64)
    return pair_weights ? launch_prefill_d<64, true>(a, items, n_items, s) : launch_prefill_d<64, false>(a, items, n_items, s);
  return hipErrorInvalidValue;
}
