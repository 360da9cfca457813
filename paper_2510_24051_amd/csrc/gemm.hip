// bf16 MFMA GEMMs  C[M, N] = A[M, K] x W[N, K]^T  with fused epilogues.
//
//   gemm_skinny : M <= 256 (decode batches, LM head).  HBM-bound on the weight stream: every wave owns one
//                 32-column block of W and reads its tiles straight from global memory into MFMA B operands
//                 (each load is 1 KiB contiguous thanks to the tiled weight layout); the activation tile is
//                 shared by the workgroup through LDS.  K is split across gridDim.y when N alone gives too
//                 few workgroups; partial sums go to a workspace and a second kernel applies the epilogue.
//   gemm_large  : M > 256 (prefill).  MFMA-bound: 256x256x64 workgroup tile, 8 waves of 128x64, LDS double
//                 buffering, swizzled A tile, W tile kept in operand order.
#include <algorithm>
#include <type_traits>

#include "internal.h"

// ------------------------------------------------------------------------------------------------
// epilogue on one 32x32 accumulator tile (rows m0.., columns n0..), see mfma32 for the lane layout
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

// Loads are batched ahead of the stores (ids, then residual values, then all stores) so that a tile costs
// three dependent memory round trips instead of one per element.
// FULL: all 32 rows of the tile exist (the caller's uniform test), so no per-row predicates are needed; with them
// every element is its own predicated block and the loads cannot be batched.
// NT: non-temporal stores (see gemm_skinny_kernel).
template <int MODE, bool FULL = false, bool NT = false>
__device__ __forceinline__ void epi_tile(const EpiArgs& e, const f32x16& acc, const f32x16& acc2, int m0, int n0,
                                         int M_rows, int N, int lane) {
  const int M = FULL ? 0x7fffffff : M_rows;
  const int n = n0 + (lane & 31);
  const int g = lane >> 5;
  if (n >= N) return;
  auto st = [](auto* p, auto v) {
    if (NT) store_nt(p, v);
    else *p = v;
  };
  int rows[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) rows[v] = m0 + (v >> 2) * 8 + g * 4 + (v & 3);
  if (MODE == EPI_STORE_BF16) {
    bf16_t* out = reinterpret_cast<bf16_t*>(e.out);
#pragma unroll
    for (int v = 0; v < 16; ++v)
      if (rows[v] < M) st(out + (int64_t)rows[v] * e.ldo + n, f32_to_bf16(acc[v]));
  } else if (MODE == EPI_STORE_F32) {
    float* out = reinterpret_cast<float*>(e.out);
#pragma unroll
    for (int v = 0; v < 16; ++v)
      if (rows[v] < M) st(out + (int64_t)rows[v] * e.ldo + n, acc[v]);
  } else if (MODE == EPI_SWIGLU) {  // acc = gate block, acc2 = up block; n0 is the gate block's packed column
    bf16_t* out = reinterpret_cast<bf16_t*>(e.out);
    const int nc = (n0 >> 1) + (lane & 31);
#pragma unroll
    for (int v = 0; v < 16; ++v)
      if (rows[v] < M) st(out + (int64_t)rows[v] * e.ldo + nc, f32_to_bf16(silu_f(acc[v]) * acc2[v]));
  } else if (MODE == EPI_RESID_EMBED) {
    float r[16];
    if (e.resid != nullptr) {  // wide residual stream of an inner layer
#pragma unroll
      for (int v = 0; v < 16; ++v) r[v] = rows[v] < M ? e.resid[(int64_t)rows[v] * e.H + n] : 0.f;
    } else {
      int id[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) id[v] = rows[v] < M ? e.ids[rows[v]] : 0;
#pragma unroll
      for (int v = 0; v < 16; ++v) r[v] = bf16_to_f32(e.embeds[(int64_t)id[v] * e.H + n]);
    }
    float* out = reinterpret_cast<float*>(e.out);
#pragma unroll
    for (int v = 0; v < 16; ++v)
      if (rows[v] < M) st(out + (int64_t)rows[v] * e.ldo + n, r[v] + acc[v]);
  } else if (MODE == EPI_RESID_OUT) {
    float r[16];
    if (e.out != nullptr) {  // inner layer: the sum stays wide and feeds the next layer
#pragma unroll
      for (int v = 0; v < 16; ++v) r[v] = rows[v] < M ? e.resid[(int64_t)rows[v] * e.H + n] : 0.f;
      float* out = reinterpret_cast<float*>(e.out);
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (rows[v] < M) st(out + (int64_t)rows[v] * e.ldo + n, r[v] + acc[v]);
    } else {
      int id[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) id[v] = rows[v] < M ? e.ids[rows[v]] : -1;
#pragma unroll
      for (int v = 0; v < 16; ++v) r[v] = id[v] >= 0 ? e.resid[(int64_t)rows[v] * e.H + n] : 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (id[v] >= 0) st(e.embeds + (int64_t)id[v] * e.H + n, f32_to_bf16(r[v] + acc[v]));
    }
  }
}

// ------------------------------------------------------------------------------------------------
// gemm_skinny
// ------------------------------------------------------------------------------------------------
#define SK_BK 128  // contraction elements per main-loop iteration (8 MFMA steps)
#define SK_MAX_SPLITS 8

// WAVES: waves per workgroup.  KS: the contraction is split KS ways INSIDE the workgroup (unsplit gate/up at widths
// that give too few waves otherwise): waves w and w + WAVES / KS own the same column block and each takes a K-th of
// the contraction, with an activation tile of its own per iteration; the sums meet through LDS at the end, so twice
// as many waves stream weights and no partial sums leave the workgroup.
template <int MB, int MODE, bool PARTIAL, int NBW, int WAVES = 4, int KS = 1>
__global__ __launch_bounds__(WAVES * 64) void gemm_skinny_kernel(const bf16_t* __restrict__ A, int lda, int M,
                                                          const bf16_t* __restrict__ Wp, int N, int NB, int K,
                                                          int iters_per_split, EpiArgs epi, float* __restrict__ part) {
  // Non-temporal stores for what is written just before a kernel that streams from HBM for a long time: the QKV sums
  // (a small rotary kernel, then decode attention) and the LM head's own logits (33 MB at 64 rows, which otherwise
  // compete with its weight stream: 205 -> 193 us).  The other products are followed by a small kernel that reads
  // what they wrote at once, and that one is a microsecond or two slower when the lines have left the caches.
  constexpr bool SK_NT = MODE == EPI_STORE_BF16 || MODE == EPI_STORE_F32 || (PARTIAL && MODE == EPI_RESID_OUT);
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem_raw);  // [2][KS][MB*32][SK_BK], 16-byte chunks swizzled by row
  static_assert(KS == 1 || (!PARTIAL && WAVES % KS == 0), "the in-workgroup split replaces the split across workgroups");
  constexpr int BM = MB * 32;
  constexpr int NT = WAVES * 64;
  constexpr int WPS = WAVES / KS;            // waves per K slice
  constexpr int A_SLICE = BM * SK_BK;        // elements of one slice's activation tile
  constexpr int A_ELEMS = KS * A_SLICE;      // elements of one stage
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ks = wave / WPS;                 // this wave's K slice
  const int KB = K / 16;
  const int total_iters = (K + SK_BK - 1) / SK_BK;
  // With KS > 1 the host launches one workgroup per column group over the whole contraction, whose iteration count
  // is a multiple of KS: slice s covers iterations s * it1 .. (s + 1) * it1 and `it` below counts within the slice.
  const int it0 = KS > 1 ? 0 : blockIdx.y * iters_per_split;
  const int it1 = KS > 1 ? total_iters / KS : min(total_iters, it0 + iters_per_split);
  const int slice_it0 = KS > 1 ? ks * it1 : 0;  // first global iteration of this wave's slice
  // a wave owns NBW adjacent 32-column blocks (SWIGLU: a gate/up pair)
  int nb0 = (blockIdx.x * WPS + wave % WPS) * NBW;
  const bool wave_active = nb0 < NB;
  if (!wave_active) nb0 = 0;  // keep loads in bounds; results are dropped

  f32x16 acc[NBW][MB];
#pragma unroll
  for (int j = 0; j < NBW; ++j)
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[j][i][v] = 0.f;

  // A tile loader: BM rows x 16 chunks (16 B) per iteration; chunk c of row r is stored at chunk (c ^ (r & 15))
  constexpr int A_CHUNKS = KS * BM * 16;     // the tiles of all slices, slice by slice
  constexpr int A_PER_THREAD = (A_CHUNKS + NT - 1) / NT;
  // The activation chunks travel in the same ring of three register sets as the weights, requested two iterations
  // ahead and stored to LDS one iteration ahead: the memory counter completes in order, so waiting for the chunks
  // of iteration it + 1 also waits for every load requested before them; with the chunks requested in the
  // previous step, the weights of two iterations stay in flight across that wait instead of one.  Only for several
  // row blocks of one column block per wave (64-row layer products: 0.244 -> 0.239 ms per forward call): with one
  // row block the extra registers cost the third wave per SIMD, and with two column blocks per wave (LM head) the
  // kernel got 2-3% slower.
  constexpr bool A_RING = MB >= 2 && NBW == 1 && (KS == 1 || WAVES >= 8);  // (few chunks per thread: the ring still fits two waves per SIMD)
  constexpr int A_SETS = A_RING ? 3 : 1;
  u32x4 areg[A_SETS][A_PER_THREAD];
  // Loads always read an in-bounds address (row and k clamped); chunks outside the matrix are zeroed when the
  // registers are stored to LDS, so no register is written while an earlier load into it could be pending.
  auto load_a = [&](int it, const int slot_ring) {
    const int slot = A_RING ? slot_ring : 0;
#pragma unroll
    for (int j = 0; j < A_PER_THREAD; ++j) {
      const int c = min(tid + j * NT, A_CHUNKS - 1);
      const int sl = c / (BM * 16), cc = c % (BM * 16);
      const int r = min(cc >> 4, M - 1), kc = cc & 15;
      const int k = min(((KS > 1 ? sl * it1 : 0) + it) * SK_BK + kc * 8, K - 8);
      areg[slot][j] = *reinterpret_cast<const u32x4*>(A + (int64_t)r * lda + k);
    }
  };
  auto store_a = [&](int buf, int it, const int slot_ring) {
    const int slot = A_RING ? slot_ring : 0;
#pragma unroll
    for (int j = 0; j < A_PER_THREAD; ++j) {
      const int c = tid + j * NT;
      const int sl = c / (BM * 16), cc = c % (BM * 16);
      const int r = cc >> 4, kc = cc & 15;
      const bool inside = r < M && ((KS > 1 ? sl * it1 : 0) + it) * SK_BK + kc * 8 < K;
      if (c < A_CHUNKS)
        *reinterpret_cast<u32x4*>(As + buf * A_ELEMS + sl * A_SLICE + r * SK_BK + ((kc ^ (r & 15)) << 3)) =
            inside ? areg[slot][j] : u32x4{0, 0, 0, 0};
    }
  };
  bf16x8 breg[3][NBW][8];  // ring of three register sets: the weights of the next two iterations are in flight
  auto load_b = [&](int it, const int slot) {
#pragma unroll
    for (int j = 0; j < NBW; ++j)
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        int kb = (slice_it0 + it) * 8 + s;
        kb = kb < KB ? kb : KB - 1;  // tail steps read a valid tile; their A operand is zero
        const int nbj = nb0 + j < NB ? nb0 + j : NB - 1;  // a missing second block re-reads a valid one
        breg[slot][j][s] = load_nt(reinterpret_cast<const bf16x8*>(Wp + packed_tile_offset(nbj, kb, KB) + lane * 8));  // read once
      }
  };

  // One main-loop iteration; SLOT is the register set holding this iteration's W operands (compile-time so
  // the operand arrays stay in registers).  The barrier carries no memory fence (a fence would make the compiler
  // drain every outstanding load, i.e. the weights requested two iterations ahead): only the LDS stores of the
  // next activation tile have to be visible to the other waves, hence the explicit wait for LDS operations.
  auto step = [&](auto slot_c, int it) {
    constexpr int SLOT = decltype(slot_c)::value;
    const int cur = (it - it0) & 1;
    const bool more = it + 1 < it1;
    if (!A_RING && more) load_a(it + 1, 0);
    if (it + 2 < it1) {
      if (A_RING) load_a(it + 2, (SLOT + 2) % 3);
      load_b(it + 2, (SLOT + 2) % 3);
    }
    const bf16_t* Ab = As + cur * A_ELEMS + ks * A_SLICE;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const int kc = s * 2 + (lane >> 5);
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        const int r = i * 32 + (lane & 31);
        bf16x8 af = *reinterpret_cast<const bf16x8*>(Ab + r * SK_BK + ((kc ^ (r & 15)) << 3));
#pragma unroll
        for (int j = 0; j < NBW; ++j) acc[j][i] = mfma32(af, breg[SLOT][j][s], acc[j][i]);
      }
    }
    if (more) store_a(cur ^ 1, it + 1, (SLOT + 1) % 3);
    PIE_S_WAIT_LGKMCNT0();
    wg_barrier();
  };
  if (it0 < it1) {
    load_a(it0, 0);
    load_b(it0, 0);
    if (it0 + 1 < it1) {
      if (A_RING) load_a(it0 + 1, 1);
      load_b(it0 + 1, 1);
    }
    store_a(0, it0, 0);  // waits for the oldest loads only
  }
  PIE_S_WAIT_LGKMCNT0();
  wg_barrier();
  for (int it = it0; it < it1; it += 3) {
    step(std::integral_constant<int, 0>{}, it);
    if (it + 1 < it1) step(std::integral_constant<int, 1>{}, it + 1);
    if (it + 2 < it1) step(std::integral_constant<int, 2>{}, it + 2);
  }
  if constexpr (!PARTIAL && MODE == EPI_SWIGLU && NBW == 1) {
    // One block per wave: the gate block sits in the even waves, its up block in the wave after it, which hands
    // its sums over through LDS (the activation stages are free once the main loop has passed its last barrier).
    float* xch = reinterpret_cast<float*>(smem_raw);  // [WPS / 2 pairs][MB][16][64]
    if constexpr (KS > 1) {
      // the slices' sums first: slices 1.. leave theirs behind the exchange area, slice 0 adds them in slice order
      float* red = xch + (WPS / 2) * MB * 16 * 64;  // [KS - 1][WPS][MB][16][64]
      if (ks > 0) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) red[((((ks - 1) * WPS + wave % WPS) * MB + i) * 16 + v) * 64 + lane] = acc[0][i][v];
      }
      __syncthreads();
      if (ks == 0) {
#pragma unroll
        for (int sl = 1; sl < KS; ++sl)
#pragma unroll
          for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[0][i][v] += red[((((sl - 1) * WPS + wave) * MB + i) * 16 + v) * 64 + lane];
      }
    }
    const int pair = (wave % WPS) >> 1;
    if ((wave & 1) && ks == 0) {
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) xch[((pair * MB + i) * 16 + v) * 64 + lane] = acc[0][i][v];
    }
    __syncthreads();
    if (!(wave & 1) && ks == 0 && wave_active) {
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        f32x16 up;
#pragma unroll
        for (int v = 0; v < 16; ++v) up[v] = xch[((pair * MB + i) * 16 + v) * 64 + lane];
        epi_tile<MODE, false, SK_NT>(epi, acc[0][i], up, i * 32, nb0 * 32, M, NB * 32, lane);
      }
    }
    return;
  }
  if (!wave_active) return;
  if (PARTIAL) {
    // raw partial sums: part[split][m][n_packed]
    float* P = part + (int64_t)blockIdx.y * M * (NB * 32);
#pragma unroll
    for (int j = 0; j < NBW; ++j)
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int m = i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
          if (m < M && nb0 + j < NB) {
            float* dst = P + (int64_t)m * (NB * 32) + (nb0 + j) * 32 + (lane & 31);
            if (SK_NT) store_nt(dst, acc[j][i][v]);
            else *dst = acc[j][i][v];
          }
        }
  } else {
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      if (MODE == EPI_SWIGLU) {
        epi_tile<MODE, false, SK_NT>(epi, acc[0][i], acc[NBW - 1][i], i * 32, nb0 * 32, M, NB * 32, lane);
      } else {
#pragma unroll
        for (int j = 0; j < NBW; ++j)
          if (nb0 + j < NB) epi_tile<MODE, false, SK_NT>(epi, acc[j][i], acc[j][i], i * 32, (nb0 + j) * 32, M, N, lane);
      }
    }
  }
}

// Sum split-K partials and apply the epilogue.  One thread per four consecutive output columns (SWIGLU: four
// gate/up pairs); all column counts are multiples of 32, so the four never straddle a 32-column block.
template <int MODE>
__global__ void splitk_epilogue_kernel(const float* __restrict__ part, int splits, int M, int N, int NP, EpiArgs e) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int cols = (MODE == EPI_SWIGLU) ? NP / 2 : N;
  const int cols4 = cols / 4;
  if (idx >= (int64_t)M * cols4) return;
  const int m = (int)(idx / cols4), c = (int)(idx % cols4) * 4;
  // partial sums are added in split order; eight loads are requested together so that the few threads of a
  // small batch still keep enough bytes in flight
  auto total = [&](int n) {
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    const float* p = part + (int64_t)m * NP + n;
    const int64_t stride = (int64_t)M * NP;
    int k = 0;
    for (; k + 8 <= splits; k += 8) {
      f32x4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const f32x4*>(p + (k + u) * stride);
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; k < splits; ++k) s += *reinterpret_cast<const f32x4*>(p + k * stride);
    return s;
  };
  auto store_bf16x4 = [](bf16_t* dst, const f32x4& v) {
    bf16x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = f32_to_bf16(v[i]);
    *reinterpret_cast<bf16x4*>(dst) = o;
  };
  if (MODE == EPI_SWIGLU) {
    const int ng = (c >> 5) * 64 + (c & 31);  // gate columns in packed order; the up columns are 32 further
    const f32x4 g = total(ng), u = total(ng + 32);
    f32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = silu_f(g[i]) * u[i];
    store_bf16x4(reinterpret_cast<bf16_t*>(e.out) + (int64_t)m * e.ldo + c, r);
  } else {
    f32x4 x = total(c);
    if (MODE == EPI_STORE_BF16) {
      store_bf16x4(reinterpret_cast<bf16_t*>(e.out) + (int64_t)m * e.ldo + c, x);
    } else if (MODE == EPI_STORE_F32) {
      *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(e.out) + (int64_t)m * e.ldo + c) = x;
    } else if (MODE == EPI_RESID_EMBED) {
      if (e.resid != nullptr) {
        x += *reinterpret_cast<const f32x4*>(e.resid + (int64_t)m * e.H + c);
      } else {
        const bf16x4 r = *reinterpret_cast<const bf16x4*>(e.embeds + (int64_t)e.ids[m] * e.H + c);
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] += bf16_to_f32(r[i]);
      }
      *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(e.out) + (int64_t)m * e.ldo + c) = x;
    } else if (MODE == EPI_RESID_OUT) {
      const f32x4 y = x + *reinterpret_cast<const f32x4*>(e.resid + (int64_t)m * e.H + c);
      if (e.out != nullptr) {
        *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(e.out) + (int64_t)m * e.ldo + c) = y;
      } else {
        const int id = e.ids[m];
        if (id >= 0) store_bf16x4(e.embeds + (int64_t)id * e.H + c, y);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// gemm_large
// ------------------------------------------------------------------------------------------------
#define LG_BM 256
#define LG_BN 256
#define LG_BK 64
#define TILED_MIN_KTS 8  // fewest k tiles a split of the tiled kernel takes

template <int MODE>
__global__ __launch_bounds__(512) void gemm_large_kernel(const bf16_t* __restrict__ A, int lda, int M,
                                                         const bf16_t* __restrict__ Wp, int N, int NB, int K,
                                                         EpiArgs epi) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t* As = reinterpret_cast<bf16_t*>(smem_raw);       // [2][256 rows][64], chunk c of row r at c ^ (r & 7)
  bf16_t* Bs = As + 2 * LG_BM * LG_BK;                    // [2][8 blocks][4 k-steps][512], operand order
  constexpr int TILE = LG_BM * LG_BK;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;  // wave tile: rows wm*128.., columns wn*64..
  const int KB = K / 16;
  const int m0 = blockIdx.y * LG_BM;
  const int nb0 = blockIdx.x * (LG_BN / 32);
  const int KT = (K + LG_BK - 1) / LG_BK;

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  u32x4 ra[4], rb[4];
  auto load_g = [&](int kt) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int c = tid + j * 512;
      int r = c >> 3, kc = c & 7;
      int gr = m0 + r;
      gr = gr < M ? gr : M - 1;  // rows past M read a valid row; their results are never stored
      int k = kt * LG_BK + kc * 8;
      u32x4 v = {0, 0, 0, 0};
      if (k < K) v = *reinterpret_cast<const u32x4*>(A + (int64_t)gr * lda + k);
      ra[j] = v;
      // W: chunk c -> block c / 256, 16-byte piece c % 256 of that block's 4 consecutive k-tiles
      int nbl = c >> 8, w = c & 255;
      int nb = nb0 + nbl;
      nb = nb < NB ? nb : NB - 1;
      int kb = kt * 4 + (w >> 6);
      u32x4 wv = {0, 0, 0, 0};
      if (kb < KB) wv = *reinterpret_cast<const u32x4*>(Wp + packed_tile_offset(nb, kb, KB) + (w & 63) * 8);
      rb[j] = wv;
    }
  };
  auto store_s = [&](int buf) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int c = tid + j * 512;
      int r = c >> 3, kc = c & 7;
      *reinterpret_cast<u32x4*>(As + buf * TILE + r * LG_BK + ((kc ^ (r & 7)) << 3)) = ra[j];
      *reinterpret_cast<u32x4*>(Bs + buf * TILE + c * 8) = rb[j];
    }
  };

  load_g(0);
  store_s(0);
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < KT;
    if (more) load_g(kt + 1);
    const bf16_t* Ab = As + cur * TILE;
    const bf16_t* Bb = Bs + cur * TILE;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bf16x8 af[4], bfr[2];
      const int kc = s * 2 + (lane >> 5);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int r = wm * 128 + i * 32 + (lane & 31);
        af[i] = *reinterpret_cast<const bf16x8*>(Ab + r * LG_BK + ((kc ^ (r & 7)) << 3));
      }
#pragma unroll
      for (int j = 0; j < 2; ++j)
        bfr[j] = *reinterpret_cast<const bf16x8*>(Bb + ((wn * 2 + j) * 4 + s) * 512 + lane * 8);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma32(af[i], bfr[j], acc[i][j]);
    }
    if (more) store_s(cur ^ 1);
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int mt = m0 + wm * 128 + i * 32;
    if (MODE == EPI_SWIGLU) {
      int nb = nb0 + wn * 2;
      if (nb < NB) epi_tile<MODE>(epi, acc[i][0], acc[i][1], mt, nb * 32, M, NB * 32, lane);
    } else {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        int nb = nb0 + wn * 2 + j;
        if (nb < NB) epi_tile<MODE>(epi, acc[i][j], acc[i][j], mt, nb * 32, M, N, lane);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// gemm_large, asynchronous-copy version (K a multiple of 64)
//
// Same 256x256x64 tile and 8 waves of 128x64 as above.  The activation tile is copied global -> LDS by direct-to-LDS
// loads (no VGPR staging, no LDS store instructions): each wave instruction moves 1 KiB and the rows land
// pre-swizzled (16-byte chunk c of row r at position c ^ ((r >> 1) & 7), conflict-free for the 64-bank LDS when 16
// consecutive rows read the same chunk); three stages as separate arrays (the compiler's wait counters then know
// which copy a read may alias), copies two k steps ahead, one fence-free barrier per k step.
// The weight operands do not pass through LDS: a wave reads the tiles of its two column blocks straight from
// global memory into MFMA B operands (the tiled weight layout makes each a contiguous 1 KiB load; the two waves
// that share a column block meet in the vector cache), one k step ahead, refilling each register set right after
// the MFMAs that consumed it.  Why: with both operands in LDS a 128x64 wave tile issues and waits for 6 LDS reads
// per 8 MFMAs, without the weights 4, and every instruction issued beside the MFMAs takes matrix time (LDS bandwidth
// itself is not short: 240-250 bytes per clock and compute unit with many reads in flight, the kernel uses a fifth
// of it).  The matrix pipe went from 62% to 72% busy, of which the lower clock under the higher load gives back a
// part (8320 x 28672 x 4096: 1.70 -> 1.58 ms on one box).
// Workgroup ids are remapped so that each XCD (id % 8) works on a contiguous range of a grouped tile order (8 row
// tiles per group) and its L2 sees a few activation and weight panels at a time.
// ------------------------------------------------------------------------------------------------
// BM = 256, or 128 for products of at most 128 rows (half the accumulators and half the activation copies per wave).
template <int MODE, bool PARTIAL, int BM>
__global__ __launch_bounds__(512) void gemm_large_async_kernel(const bf16_t* __restrict__ A, int lda, int M,
                                                               const bf16_t* __restrict__ Wp, int N, int NB, int K,
                                                               EpiArgs epi, int tiles_m, int tiles_n,
                                                               int kts_per_split, float* __restrict__ part) {
  static_assert(BM == 256 || BM == 128, "tile height");
  constexpr int MI = BM / 64;  // 32-row accumulator blocks per wave, and activation copy instructions per wave
  __shared__ __align__(16) bf16_t As0[BM * LG_BK], As1[BM * LG_BK], As2[BM * LG_BK];  // three activation stages
  constexpr int GROUP_M = 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  const int KB = K / 16, KT = K / LG_BK;
  // split K: workgroup row blockIdx.y takes k tiles [kt0, kt1)
  // Non-temporal stores for the logits and for the partial sums of the down projection, the last product before the
  // LM head (see gemm_skinny_kernel; LM head at 128 rows 259 -> 238 us, at 256 rows 278 -> 262 us).  The partial sums
  // of the QKV product are stored plainly here: at 65 to 256 rows the rotary step that sums them loses what the
  // attention kernel gains.
  constexpr bool LG_NT = MODE == EPI_STORE_F32 || (PARTIAL && MODE == EPI_RESID_OUT) || (!PARTIAL && MODE == EPI_SWIGLU);
  const int kt0 = PARTIAL ? blockIdx.y * kts_per_split : 0;
  const int kt1 = PARTIAL ? min(KT, kt0 + kts_per_split) : KT;
  int pid = blockIdx.x;
  const int ntiles = tiles_m * tiles_n;
  if (ntiles % 8 == 0) pid = (pid & 7) * (ntiles / 8) + (pid >> 3);
  int tm, tn;
  {
    const int width = GROUP_M * tiles_n;
    const int first_m = (pid / width) * GROUP_M;
    const int gsz = min(tiles_m - first_m, GROUP_M);
    tm = first_m + (pid % width) % gsz;
    tn = (pid % width) / gsz;
  }
  const int m0 = tm * BM, nb0 = tn * (LG_BN / 32);

  f32x16 acc[MI][2];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  {
#if __HIP_DEVICE_COMPILE__  // (the buffer-descriptor builtins exist for the device target only)
    // Both operands are addressed through buffer descriptors (base in scalar registers, a 32-bit byte offset per
    // lane, the k step as a scalar offset): a request is one instruction without 64-bit address arithmetic, reads
    // past the end return zeros, and the direct-to-LDS copies are buffer loads, not global (flat-encoded) loads:
    // with those in flight the compiler waits for all outstanding vector memory operations before every use of a
    // register that a load returns, which would drain the weight loads requested ahead at every step.
    constexpr int RSRC_FLAGS = 0x00020000;  // raw dword buffer, gfx9 family
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(A), 0, (int)(((int64_t)(M - 1) * lda + K) * 2), RSRC_FLAGS);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<bf16_t*>(Wp), 0, (int)((int64_t)NB * 32 * K * 2), RSRC_FLAGS);
    // copy instruction j = wave * MI + jj of a stage covers LDS bytes [j KiB, (j + 1) KiB): rows j*8 .. j*8+7 of
    // the tile, lane -> row j*8 + lane/8, stored chunk lane%8
    int aoff[MI], woff[2];  // byte offsets of this lane's pieces at k step 0
#pragma unroll
    for (int jj = 0; jj < MI; ++jj) {
      const int r = (wave * MI + jj) * 8 + (lane >> 3);
      const int kc = (lane & 7) ^ ((r >> 1) & 7);
      int gr = m0 + r;
      gr = gr < M ? gr : M - 1;  // rows past M re-read a valid row; their results are never stored
      aoff[jj] = (int)(((int64_t)gr * lda + kc * 8) * 2);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      int nb = nb0 + wn * 2 + j;
      nb = nb < NB ? nb : NB - 1;  // a column block past the matrix re-reads a valid one; its results are dropped
      woff[j] = (int)((packed_tile_offset(nb, 0, KB) + lane * 8) * 2);
    }
    u32x4 wreg[4][2];  // the weight operands of one k step: [16-wide contraction step][column block]
    auto issue_a = [&](bf16_t* As, int kt) {
      const int k = kt < kt1 ? kt : kt1 - 1;  // past the end: a copy nobody reads, so that the wait counts stay uniform
#pragma unroll
      for (int jj = 0; jj < MI; ++jj)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, (__attribute__((address_space(3))) void*)(As + (wave * MI + jj) * 512),
                                                 16, aoff[jj], k * (LG_BK * 2), 0, 0);
    };
    auto load_w = [&](int kt, const int s) {
      const int k = kt < kt1 ? kt : kt1 - 1;
#pragma unroll
      for (int j = 0; j < 2; ++j) wreg[s][j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, woff[j], (k * 4 + s) * 1024, 0);
    };
    auto load_a = [&](const bf16_t* As, int s, bf16x8 (&af)[MI]) {
      const int kc = s * 2 + (lane >> 5);
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const int r = wm * (BM / 2) + i * 32 + (lane & 31);
        af[i] = *reinterpret_cast<const bf16x8*>(As + r * LG_BK + ((kc ^ ((r >> 1) & 7)) << 3));
      }
    };
    // One k step on stage Acur; the copy of k step kt + 2 goes to Afill (read last in k step kt - 1, which every wave
    // has left).  The step's barrier sits before its last 16-wide contraction step instead of at its end: by then a
    // wave has read everything it needs from Acur, so after the barrier the first operands of the next k step can be
    // read from Anext while the last MFMAs of this one run, and no step starts with the matrix cores waiting for
    // LDS.  Vector memory operations complete in order: at the barrier the newest MI + 6 (the copy issued at the top
    // of the step and the weight loads of its first three contraction steps) may still be in flight, everything
    // older has arrived, in particular this wave's part of the activation tile of k step kt + 1.
    bf16x8 af[2][MI];
    auto step = [&](const bf16_t* Acur, const bf16_t* Anext, bf16_t* Afill, int kt) {
      issue_a(Afill, kt + 2);
      __builtin_amdgcn_sched_barrier(0);  // the copies go out first: the wait counts rely on the request order
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        if (s + 1 < 4) {
          load_a(Acur, s + 1, af[(s + 1) & 1]);
        } else {
          PIE_S_WAIT_LGKMCNT0();  // this wave's last reads of Acur have returned
          PIE_S_WAIT_VMCNT(MI + 6);
          wg_barrier();
          load_a(Anext, 0, af[0]);
        }
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            Pack16 w;
            w.u = wreg[s][j];
            acc[i][j] = mfma32(af[s & 1][i], w.h, acc[i][j]);
          }
        load_w(kt + 1, s);  // refill the registers just consumed with the next k step's weights
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    issue_a(As0, kt0);
    issue_a(As1, kt0 + 1);
#pragma unroll
    for (int s = 0; s < 4; ++s) load_w(kt0, s);
    PIE_S_WAIT_VMCNT(MI + 8);  // the first activation tile has arrived
    wg_barrier();
    load_a(As0, 0, af[0]);
    int kt = kt0;
    for (; kt + 3 <= kt1; kt += 3) {  // whole revolutions of the three stages; the one or two steps left over follow
      step(As0, As1, As2, kt);
      step(As1, As2, As0, kt + 1);
      step(As2, As0, As1, kt + 2);
    }
    if (kt < kt1) {
      step(As0, As1, As2, kt);
      if (kt + 1 < kt1) step(As1, As2, As0, kt + 1);
    }
    PIE_S_WAIT_VMCNT(0);  // the surplus copies of the last steps land before the workgroup gives up its LDS
#endif
  }
  if (PARTIAL) {
    // raw partial sums: part[split][m][n_packed]
    const int NP = NB * 32;
    float* P = part + (int64_t)blockIdx.y * M * NP;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int nb = nb0 + wn * 2 + j;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = m0 + wm * (BM / 2) + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
          if (m < M && nb < NB) {
            float* dst = P + (int64_t)m * NP + nb * 32 + (lane & 31);
            if (LG_NT) store_nt(dst, acc[i][j][v]);
            else *dst = acc[i][j][v];
          }
        }
      }
    return;
  }
  // row tiles that lie wholly inside the matrix (all of them except in a ragged last row block) take the
  // epilogue without per-row predicates
  auto epilogue = [&](auto full_c) {
    constexpr bool FULL = decltype(full_c)::value;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int mt = m0 + wm * (BM / 2) + i * 32;
      if (MODE == EPI_SWIGLU) {
        int nb = nb0 + wn * 2;
        if (nb < NB) epi_tile<MODE, FULL, LG_NT>(epi, acc[i][0], acc[i][1], mt, nb * 32, M, NB * 32, lane);
      } else {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          int nb = nb0 + wn * 2 + j;
          if (nb < NB) epi_tile<MODE, FULL, LG_NT>(epi, acc[i][j], acc[i][j], mt, nb * 32, M, N, lane);
        }
      }
    }
  };
  const bool rows_full = m0 + wm * (BM / 2) + MI * 32 <= M;
  if constexpr (MODE == EPI_RESID_EMBED || MODE == EPI_RESID_OUT) {
    // Residual epilogues of full row tiles, pipelined over the wave's 2 * MI accumulator tiles: the Embed ids of
    // all its rows are read first (one round trip), then the residual values of tile t + 1 are requested before
    // tile t is stored, so a tile no longer costs two or three dependent round trips of its own.
    if (rows_full && N % 32 == 0) {
      const bool by_id = MODE == EPI_RESID_EMBED ? epi.resid == nullptr : epi.out == nullptr;
      const int g = lane >> 5;
      const int mw = m0 + wm * (BM / 2) + g * 4;
      auto row_of = [&](int i, int v) { return mw + i * 32 + (v >> 2) * 8 + (v & 3); };
      auto run = [&](auto by_id_c) {
        constexpr bool BY_ID = decltype(by_id_c)::value;
        int id[MI][16];
        if (BY_ID) {
#pragma unroll
          for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) id[i][v] = epi.ids[row_of(i, v)];
        }
        float r[2][16];
        auto col_of = [&](int t) { return (nb0 + wn * 2 + (t & 1)) * 32 + (lane & 31); };
        auto fetch = [&](int t, float (&dst)[16]) {
          const int i = t >> 1, n = col_of(t);
          if (n >= N) return;  // uniform: a column block past the matrix
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            if (MODE == EPI_RESID_EMBED && BY_ID) dst[v] = bf16_to_f32(epi.embeds[(int64_t)id[i][v] * epi.H + n]);
            else dst[v] = epi.resid[(int64_t)row_of(i, v) * epi.H + n];
          }
        };
        auto put = [&](int t, const float (&src)[16]) {
          const int i = t >> 1, j = t & 1, n = col_of(t);
          if (n >= N) return;
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const float y = src[v] + acc[i][j][v];
            if (MODE == EPI_RESID_OUT && BY_ID) {
              // (non-temporal: the output Embeds are the last thing written before the LM head streams its weights:
              // 241 -> 219 us at 8320 rows; the fp32 sums of the output projection below lose 9 us that way)
              if (id[i][v] >= 0) store_nt(epi.embeds + (int64_t)id[i][v] * epi.H + n, f32_to_bf16(y));
            } else if (MODE == EPI_RESID_OUT) {
              store_nt(reinterpret_cast<float*>(epi.out) + (int64_t)row_of(i, v) * epi.ldo + n, y);
            } else {
              reinterpret_cast<float*>(epi.out)[(int64_t)row_of(i, v) * epi.ldo + n] = y;
            }
          }
        };
        fetch(0, r[0]);
#pragma unroll
        for (int t = 0; t < 2 * MI; ++t) {
          if (t + 1 < 2 * MI) fetch(t + 1, r[(t + 1) & 1]);
          put(t, r[t & 1]);
        }
      };
      if (by_id) run(std::true_type{});
      else run(std::false_type{});
      return;
    }
  }
  if (rows_full) epilogue(std::true_type{});
  else epilogue(std::false_type{});
}

// ------------------------------------------------------------------------------------------------
// dispatch
// ------------------------------------------------------------------------------------------------
// Raises a kernel's dynamic LDS limit once per process and device (done: one bit per device), not per launch.
static hipError_t set_lds_limit_once(const void* kern, size_t bytes, uint32_t& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev >= 0 && dev < 32 && ((done >> dev) & 1u)) return hipSuccess;
  e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess && dev >= 0 && dev < 32) done |= 1u << dev;
  return e;
}

template <int MB, int MODE, int NBW, int WAVES = 4, int KS = 1>
static hipError_t run_skinny_n(const bf16_t* A, int lda, int M, const PackedWeight& W, const EpiArgs& epi, float* ws,
                               size_t ws_elems, int n_cus, hipStream_t s, int* defer, int max_splits = SK_MAX_SPLITS) {
  const int wg_n = (W.NB + (WAVES / KS) * NBW - 1) / ((WAVES / KS) * NBW);
  const int total_iters = (W.K + SK_BK - 1) / SK_BK;
  // Split K so that one round of workgroups fills the chip without spilling into a second, mostly empty round:
  // the kernel keeps `occ` workgroups per CU resident (register-limited).
  const int occ = (MB == 1 && NBW == 1) ? 3 : ((MB * NBW <= 2) ? 2 : 1);
  const int slots = n_cus * occ;
  int splits = slots / wg_n;
  if (splits > total_iters / 2) splits = total_iters / 2;
  // Every split writes an M x N fp32 partial that is read back once and then sits dirty in the caches until the
  // next weight stream pushes it out to HBM; beyond 8 splits that costs more than the extra workgroups gain
  // (c2 forward -2.5 us, c5 -8 us against 16 and 12 splits).
  if (splits > max_splits) splits = max_splits;
  // The QKV product does as well with half as many splits while three quarters of the CUs still get a workgroup
  // (8B shape at 64 rows: the same 18 us with 192 workgroups as with 384; 70B shape at 16 rows: 36 against 37 us),
  // and every split less is an M x N partial less for the rotary step to read and to be written out of the caches
  // underneath the attention kernel (8B: -1.5 and -1 us).  The output and down projections lose more than the
  // kernels after them gain (70B shape: +2 and +8 us), so they keep their splits.
  if (MODE == EPI_STORE_BF16)
    while (splits >= 4 && splits % 2 == 0 && wg_n * (splits / 2) * 4 >= n_cus * 3) splits /= 2;
  if (splits < 1) splits = 1;
  const int NP = W.NB * 32;
  while (splits > 1 && (size_t)splits * M * NP > ws_elems) --splits;
  int ips = (total_iters + splits - 1) / splits;
  splits = (total_iters + ips - 1) / ips;
  size_t smem = (size_t)2 * KS * MB * 32 * SK_BK * sizeof(bf16_t);
  dim3 grid(wg_n, splits), block(WAVES * 64);
  if (splits == 1) {
    auto kern = gemm_skinny_kernel<MB, MODE, false, NBW, WAVES, KS>;
    static uint32_t lds_set = 0;
    hipError_t e = set_lds_limit_once((const void*)kern, smem, lds_set);
    if (e != hipSuccess) return e;
    kern<<<grid, block, smem, s>>>(A, lda, M, W.data, W.N, W.NB, W.K, ips, epi, nullptr);
    return hipGetLastError();
  }
  if constexpr (KS > 1) return hipErrorInvalidValue;  // (the in-workgroup split is launched unsplit only)
  auto kern = gemm_skinny_kernel<MB, MODE, true, NBW, WAVES, 1>;
  static uint32_t lds_set_partial = 0;
  hipError_t e = set_lds_limit_once((const void*)kern, smem, lds_set_partial);
  if (e != hipSuccess) return e;
  kern<<<grid, block, smem, s>>>(A, lda, M, W.data, W.N, W.NB, W.K, ips, epi, ws);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (defer) { *defer = splits; return hipSuccess; }  // the caller's next kernel sums the partials
  const int cols = (MODE == EPI_SWIGLU) ? NP / 2 : W.N;
  int64_t total = (int64_t)M * (cols / 4);
  splitk_epilogue_kernel<MODE><<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s>>>(ws, splits, M, W.N, NP, epi);
  return hipGetLastError();
}

template <int MB, int MODE>
static hipError_t run_skinny(const bf16_t* A, int lda, int M, const PackedWeight& W, const EpiArgs& epi, float* ws,
                             size_t ws_elems, int n_cus, hipStream_t s, int* defer) {
  if constexpr (MODE == EPI_SWIGLU) {
    // Wide enough MLPs fill the chip with one block per wave and no split at all (gate and up meet through LDS):
    // no partial sums to write, read back and write out of the caches (70B shape, 16 rows: 179 -> 163 us, the
    // forward call 0.410 -> 0.389 ms).  With fewer workgroups than that (8B shape: 224 on 256 CUs) the split
    // version with a gate/up pair per wave is faster.
    if constexpr (MB <= 2) {
      if ((W.NB + 3) / 4 >= n_cus + n_cus / 2)
        return run_skinny_n<MB, MODE, 1>(A, lda, M, W, epi, ws, ws_elems, n_cus, s, defer, 1);
      // the 8B width gets there with workgroups of one pair (two waves): 448 of them; as fast as the split
      // version and without its 29 MB of partial sums (the down projection after it gains 1 us)
      if ((W.NB + 1) / 2 >= n_cus + n_cus / 2) {
        // With two row blocks a two-wave workgroup fetches as many activation bytes (through the L2) as weight
        // bytes.  Eight waves, two pairs times two K slices, share each slice's activation tile between two pairs
        // and put twice as many waves on the weight stream: 53 -> 47 us at 64 rows.  (Four waves, one pair times two
        // slices, measured the same as two; with one row block the two-wave form stays ahead.)
        if (MB == 2 && W.K % (2 * SK_BK) == 0)
          return run_skinny_n<MB, MODE, 1, 8, 2>(A, lda, M, W, epi, ws, ws_elems, n_cus, s, defer, 1);
        return run_skinny_n<MB, MODE, 1, 2>(A, lda, M, W, epi, ws, ws_elems, n_cus, s, defer, 1);
      }
    }
    return run_skinny_n<MB, MODE, 2>(A, lda, M, W, epi, ws, ws_elems, n_cus, s, defer);
  } else {
    // wide outputs (LM head): two blocks per wave halve the workgroup count and the activation reads from LDS
    if constexpr (MB <= 2)
      if ((W.NB + 3) / 4 > n_cus * (MB == 1 ? 3 : 2))
        return run_skinny_n<MB, MODE, 2>(A, lda, M, W, epi, ws, ws_elems, n_cus, s, defer);
    return run_skinny_n<MB, MODE, 1>(A, lda, M, W, epi, ws, ws_elems, n_cus, s, defer);
  }
}

// The epilogue arguments of rows m0.. of the same product.
template <int MODE>
static EpiArgs offset_rows(EpiArgs e, int m0) {
  if (MODE == EPI_STORE_BF16 || MODE == EPI_SWIGLU) e.out = reinterpret_cast<bf16_t*>(e.out) + (int64_t)m0 * e.ldo;
  if (MODE == EPI_STORE_F32 || MODE == EPI_RESID_EMBED || (MODE == EPI_RESID_OUT && e.out != nullptr))
    e.out = reinterpret_cast<float*>(e.out) + (int64_t)m0 * e.ldo;
  if ((MODE == EPI_RESID_EMBED || MODE == EPI_RESID_OUT) && e.ids != nullptr) e.ids += m0;
  if ((MODE == EPI_RESID_EMBED || MODE == EPI_RESID_OUT) && e.resid != nullptr) e.resid += (int64_t)m0 * e.H;
  return e;
}

template <int MODE>
static hipError_t run_mode(const bf16_t* A, int lda, int M, const PackedWeight& W, const EpiArgs& epi, float* ws,
                           size_t ws_elems, int n_cus, hipStream_t s, int* defer) {
  if (M <= 0) return hipSuccess;
  if (M <= 32) return run_skinny<1, MODE>(A, lda, M, W, epi, ws, ws_elems, n_cus, s, defer);
  if (M <= 64) return run_skinny<2, MODE>(A, lda, M, W, epi, ws, ws_elems, n_cus, s, defer);
  // Very wide outputs (the LM head) give the tiled kernel at least one tile per CU even with a single row
  // block; above 64 rows it beats streaming the weights past 4-8 row blocks per wave (measured at 128256 x 4096:
  // 0.26 ms for up to 256 rows against 0.30 ms at 128 rows and 0.46 ms at 256 rows).
  // the tiled kernel steps 64 contraction elements at a time and addresses both operands with 32-bit byte offsets
  const bool tiled_ok = W.K % LG_BK == 0 && (int64_t)M * lda * 2 < ((int64_t)1 << 32) &&
                        (int64_t)W.NB * 32 * W.K * 2 < ((int64_t)1 << 32);
  const bool wide = tiled_ok && (W.NB + 7) / 8 >= n_cus && M > 64;
  if (M <= 256 && !wide && tiled_ok) {
    // One row of 256-column tiles (128 rows high up to 128 rows, else 256) with K split so that the tiles fill the
    // chip once; each split keeps at least TILED_MIN_KTS k tiles, or the pipeline fill and the partial sums
    // outweigh the work.
    const int tiles_n = (W.NB + 7) / 8, KT = W.K / LG_BK, NP = W.NB * 32;
    int splits = std::max(1, n_cus / tiles_n);
    int kts = (KT + splits - 1) / splits;
    kts = std::max(kts, TILED_MIN_KTS);
    splits = (KT + kts - 1) / kts;
    if (splits > 1 && (size_t)splits * M * NP <= ws_elems) {
      if (M <= 128)
        gemm_large_async_kernel<MODE, true, 128><<<dim3(tiles_n, splits), dim3(512), 0, s>>>(
            A, lda, M, W.data, W.N, W.NB, W.K, epi, 1, tiles_n, kts, ws);
      else
        gemm_large_async_kernel<MODE, true, 256><<<dim3(tiles_n, splits), dim3(512), 0, s>>>(
            A, lda, M, W.data, W.N, W.NB, W.K, epi, 1, tiles_n, kts, ws);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
      if (defer) { *defer = splits; return hipSuccess; }
      const int cols = (MODE == EPI_SWIGLU) ? NP / 2 : W.N;
      const int64_t total = (int64_t)M * (cols / 4);
      splitk_epilogue_kernel<MODE><<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s>>>(ws, splits, M, W.N, NP, epi);
      return hipGetLastError();
    }
  }
  if (M <= 128 && !wide) return run_skinny<4, MODE>(A, lda, M, W, epi, ws, ws_elems, n_cus, s, defer);
  if constexpr (MODE != EPI_SWIGLU) {  // (eight row blocks of gate/up pairs would not fit the register file)
    if (M <= 256 && !wide) return run_skinny<8, MODE>(A, lda, M, W, epi, ws, ws_elems, n_cus, s, defer);
  }
  if (tiled_ok) {
    const int tiles_n = (W.NB + 7) / 8;
    // A ragged last row block that would open one more round of tiles (a round = one tile per CU) costs a whole
    // round for a fraction of a tile's work: those rows go through the weight-streaming kernel instead.
    const int full = M / LG_BM, ragged = M % LG_BM;
    auto rounds = [&](int tm) { return (tm * tiles_n + n_cus - 1) / n_cus; };
    if (ragged > 0 && full > 0 && (ragged <= 128 || MODE != EPI_SWIGLU) && rounds(full + 1) > rounds(full)) {
      const int M0 = full * LG_BM;
      gemm_large_async_kernel<MODE, false, 256><<<dim3(full * tiles_n), dim3(512), 0, s>>>(
          A, lda, M0, W.data, W.N, W.NB, W.K, epi, full, tiles_n, 0, nullptr);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
      return run_mode<MODE>(A + (int64_t)M0 * lda, lda, ragged, W, offset_rows<MODE>(epi, M0), ws, ws_elems, n_cus, s,
                            nullptr);
    }
    const int tiles_m = (M + LG_BM - 1) / LG_BM;
    if (M <= 128)
      gemm_large_async_kernel<MODE, false, 128><<<dim3(tiles_n), dim3(512), 0, s>>>(A, lda, M, W.data, W.N, W.NB, W.K, epi,
                                                                                   1, tiles_n, 0, nullptr);
    else
      gemm_large_async_kernel<MODE, false, 256><<<dim3(tiles_m * tiles_n), dim3(512), 0, s>>>(
          A, lda, M, W.data, W.N, W.NB, W.K, epi, tiles_m, tiles_n, 0, nullptr);
    return hipGetLastError();
  }
  auto kern = gemm_large_kernel<MODE>;
  size_t smem = (size_t)4 * LG_BM * LG_BK * sizeof(bf16_t);
  static uint32_t lds_set_large = 0;
  hipError_t e = set_lds_limit_once((const void*)kern, smem, lds_set_large);
  if (e != hipSuccess) return e;
  dim3 grid((W.NB + 7) / 8, (M + LG_BM - 1) / LG_BM), block(512);
  kern<<<grid, block, smem, s>>>(A, lda, M, W.data, W.N, W.NB, W.K, epi);
  return hipGetLastError();
}

hipError_t launch_gemm(const bf16_t* A, int lda, int M, const PackedWeight& W, const EpiArgs& epi, float* splitk_ws,
                       size_t splitk_elems, int n_cus, hipStream_t s, int* deferred_splits) {
  // Deferral is only offered where the whole product goes through one split-K launch (at most 256 rows).
  int* defer = (deferred_splits && M <= 256) ? deferred_splits : nullptr;
  if (deferred_splits) *deferred_splits = 0;
  switch (epi.mode) {
    case EPI_STORE_BF16: return run_mode<EPI_STORE_BF16>(A, lda, M, W, epi, splitk_ws, splitk_elems, n_cus, s, defer);
    case EPI_RESID_EMBED: return run_mode<EPI_RESID_EMBED>(A, lda, M, W, epi, splitk_ws, splitk_elems, n_cus, s, defer);
    case EPI_SWIGLU: return run_mode<EPI_SWIGLU>(A, lda, M, W, epi, splitk_ws, splitk_elems, n_cus, s, defer);
    case EPI_RESID_OUT: return run_mode<EPI_RESID_OUT>(A, lda, M, W, epi, splitk_ws, splitk_elems, n_cus, s, defer);
    case EPI_STORE_F32: return run_mode<EPI_STORE_F32>(A, lda, M, W, epi, splitk_ws, splitk_elems, n_cus, s, defer);
  }
  return hipErrorInvalidValue;
}
