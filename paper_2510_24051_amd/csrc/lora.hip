// LoRA adapters (forward_with_adapter): per-token low-rank updates  y += scale * B (A x)  of the layer's
// projections.  Tokens carry the adapter of their request (-1: none); the pairs of all adapters live in one
// device table indexed [adapter][layer][projection], A stored [rank_p, in] and B [out, rank_p] with the rank padded
// to a multiple of 16 by zeros.  The batch plan lists the adapted tokens grouped by adapter in tiles of 32 rows
// (row = token index, -1 = padding; one adapter per tile), so both steps are small grouped GEMMs on the matrix
// cores and A, B are read once per 32 tokens:
//   lora_down  z[row, slot, :] = A x            X rows gathered as the MFMA A operand, A's rows as the B operand,
//                                               the contraction split over the workgroup's four waves
//   lora_up    y[token, n]    += scale * B z    z (fp32) enters as a bf16 pair hi + lo, so that its rounding does
//                                               not show; y is the bf16 qkv row, the fp32 residual stream, or the
//                                               fp32 gate/up sums in the packed column order of the tiled weight
// When gate or up carry an adapter the SwiGLU product cannot be fused into the GEMM epilogue; it is taken from the
// fp32 sums by `swiglu_f32`.
#include <algorithm>

#include "internal.h"

namespace {

__device__ __forceinline__ const LoraPair& pair_of(const LoraPair* table, int ad, int n_layers, int layer, int proj) {
  return table[((int64_t)ad * n_layers + layer) * PIE_N_PROJ + proj];
}

// grid (tiles, slots, rank blocks of 32 x ksplits); z is [ksplits][rows, 3, rmax_p] fp32: with few tiles the
// contraction is also split over workgroups (partial sums that lora_up adds while it loads z), or a handful of
// workgroups would walk the whole input dimension one dependent load after the other
__global__ __launch_bounds__(256) void lora_down_kernel(const bf16_t* __restrict__ x, int ldx, int in,
                                                        const int32_t* __restrict__ rows,
                                                        const int32_t* __restrict__ tile_ad,
                                                        const LoraPair* __restrict__ table, int layer, int n_layers,
                                                        int proj0, float* __restrict__ z, int rmax_p, int ksplits) {
  __shared__ float red[4][16][64];
  const int tile = blockIdx.x, slot = blockIdx.y, rb = blockIdx.z / ksplits, ks = blockIdx.z % ksplits;
  const LoraPair p = pair_of(table, tile_ad[tile], n_layers, layer, proj0 + slot);
  if (p.A == nullptr || rb * 32 >= p.rank_p) return;  // the same for the whole workgroup
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m = lane & 31, g = lane >> 5;
  const int tok = max(rows[tile * 32 + m], 0);  // padding rows read token 0; their sums are never used
  const bf16_t* xr = x + (int64_t)tok * ldx + g * 8;
  const bf16_t* ar = p.A + (int64_t)min(rb * 32 + m, p.rank_p - 1) * in + g * 8;
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  const int steps = in / 16;  // `in` is a multiple of 32
  const int per = (steps + ksplits - 1) / ksplits;
  const int s_end = min(steps, (ks + 1) * per);
#pragma unroll 4
  for (int s = ks * per + wave; s < s_end; s += 4) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(xr + s * 16);
    const bf16x8 b = *reinterpret_cast<const bf16x8*>(ar + s * 16);
    acc = mfma32(a, b, acc);
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) red[wave][v][lane] = acc[v];
  __syncthreads();
  // wave w finishes accumulator registers 4w .. 4w+3: row (v / 4) * 8 + g * 4 + (v % 4) of the tile, column m
  const int j = rb * 32 + m;
  if (j >= p.rank_p) return;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int v = wave * 4 + q;
    const float sum = (red[0][v][lane] + red[1][v][lane]) + (red[2][v][lane] + red[3][v][lane]);
    const int row = (v >> 2) * 8 + g * 4 + (v & 3);
    z[(((int64_t)ks * gridDim.x + tile) * 32 + row) * 3 * rmax_p + slot * rmax_p + j] = sum;
  }
}

// grid (tiles, blocks of 128 output columns); a wave owns 32 columns
//   kind 0: dst bf16, column = col0 + n       (q, k or v inside the qkv rows)
//   kind 1: dst fp32, column = col0 + n       (residual stream)
//   kind 2: dst fp32, column = (n / 32) * 64 + n % 32 + col0   (gate: col0 = 0, up: col0 = 32; packed order)
//   kind 3: dst bf16 qkv rows, all three projections in one launch: out = the row length, columns [0, col0) are
//           q (projection proj, slot 0), the next kd columns k (proj + 1, slot 1), the rest v (proj + 2, slot 2)
__global__ __launch_bounds__(256) void lora_up_kernel(void* __restrict__ dst, int ld, int out, int kind, int col0,
                                                      int kd, const int32_t* __restrict__ rows,
                                                      const int32_t* __restrict__ tile_ad,
                                                      const LoraPair* __restrict__ table, int layer, int n_layers,
                                                      int proj, int slot, const float* __restrict__ z, int rmax_p,
                                                      int ksplits) {
  const int tile = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nb = blockIdx.y * 4 + wave;
  if (nb * 32 >= out) return;  // `out` is a multiple of 32; no barrier below
  const int m = lane & 31, g = lane >> 5;
  int n = nb * 32 + m, col_base = col0;
  if (kind == 3) {  // which of q, k, v this block of 32 columns belongs to (their widths are multiples of 32)
    const int seg = nb * 32 < col0 ? 0 : (nb * 32 < col0 + kd ? 1 : 2);
    col_base = seg == 0 ? 0 : (seg == 1 ? col0 : col0 + kd);
    n -= col_base;
    proj += seg;
    slot = seg;
  }
  const LoraPair p = pair_of(table, tile_ad[tile], n_layers, layer, proj);
  if (p.B == nullptr) return;
  const float* zr = z + ((int64_t)(tile * 32 + m) * 3 + slot) * rmax_p + g * 8;
  const int64_t zsplit = (int64_t)gridDim.x * 32 * 3 * rmax_p;
  const bf16_t* br = p.B + (int64_t)n * p.rank_p + g * 8;
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  for (int s = 0; s < p.rank_p / 16; ++s) {
    f32x4 z0 = {0.f, 0.f, 0.f, 0.f}, z1 = {0.f, 0.f, 0.f, 0.f};
    int k = 0;
    for (; k + 4 <= ksplits; k += 4) {  // four partial copies requested together
      f32x4 pa[4], pb[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        pa[u] = *reinterpret_cast<const f32x4*>(zr + (k + u) * zsplit + s * 16);
        pb[u] = *reinterpret_cast<const f32x4*>(zr + (k + u) * zsplit + s * 16 + 4);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) { z0 += pa[u]; z1 += pb[u]; }
    }
    for (; k < ksplits; ++k) {
      z0 += *reinterpret_cast<const f32x4*>(zr + k * zsplit + s * 16);
      z1 += *reinterpret_cast<const f32x4*>(zr + k * zsplit + s * 16 + 4);
    }
    const bf16x8 b = *reinterpret_cast<const bf16x8*>(br + s * 16);
    bf16x8 hi, lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float f = e < 4 ? z0[e] : z1[e - 4];
      hi[e] = f32_to_bf16(f);
      lo[e] = f32_to_bf16(f - bf16_to_f32(hi[e]));
    }
    acc = mfma32(hi, b, acc);
    acc = mfma32(lo, b, acc);
  }
  int tok[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) tok[v] = rows[tile * 32 + (v >> 2) * 8 + g * 4 + (v & 3)];
  const int col = kind == 2 ? (n >> 5) * 64 + (n & 31) + col0 : col_base + n;
  if (kind == 0 || kind == 3) {
    bf16_t* d = reinterpret_cast<bf16_t*>(dst) + col;
    float old[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) old[v] = tok[v] >= 0 ? bf16_to_f32(d[(int64_t)tok[v] * ld]) : 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v)
      if (tok[v] >= 0) d[(int64_t)tok[v] * ld] = f32_to_bf16(old[v] + acc[v] * p.scale);
  } else {
    float* d = reinterpret_cast<float*>(dst) + col;
    float old[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) old[v] = tok[v] >= 0 ? d[(int64_t)tok[v] * ld] : 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v)
      if (tok[v] >= 0) d[(int64_t)tok[v] * ld] = old[v] + acc[v] * p.scale;
  }
}

// act[t, i] = silu(gate) * up from fp32 sums in the packed column order (gate block, up block alternating)
__global__ __launch_bounds__(256) void swiglu_f32_kernel(const float* __restrict__ gu, int I, bf16_t* __restrict__ act,
                                                         int64_t total) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int i = (int)(idx % I);
  const int64_t t = idx / I;
  const float* row = gu + t * 2 * I;
  const int c = (i >> 5) * 64 + (i & 31);
  const float g = row[c], u = row[c + 32];
  act[idx] = f32_to_bf16(g / (1.0f + __expf(-g)) * u);
}

}  // namespace

int lora_ksplits(int n_tiles, int n_slots, int in, int rmax_p, size_t z_rows) {
  // enough workgroups to cover the chip, at least 4 contraction steps per wave, and room for the partial copies
  const int wgs = n_tiles * n_slots * ((rmax_p + 31) / 32);
  int ks = std::max(1, 256 / std::max(1, wgs));
  ks = std::min(ks, std::max(1, in / 16 / 16));
  ks = std::min<int>(ks, (int)std::max<size_t>(1, z_rows / ((size_t)n_tiles * 32)));
  return std::min(ks, 16);
}

hipError_t launch_lora_down(const bf16_t* x, int ldx, int in, int n_tiles, int n_slots, const int32_t* rows,
                            const int32_t* tile_ad, const LoraPair* table, int layer, int n_layers, int proj0, float* z,
                            int rmax_p, int ksplits, hipStream_t s) {
  if (n_tiles <= 0 || n_slots <= 0) return hipSuccess;
  if (n_slots > 3 || in % 32 != 0 || rmax_p % 16 != 0 || ksplits < 1) return hipErrorInvalidValue;
  lora_down_kernel<<<dim3(n_tiles, n_slots, ((rmax_p + 31) / 32) * ksplits), dim3(256), 0, s>>>(
      x, ldx, in, rows, tile_ad, table, layer, n_layers, proj0, z, rmax_p, ksplits);
  return hipGetLastError();
}

hipError_t launch_lora_up(void* dst, int ld, int out, int kind, int col0, int kd, int n_tiles, const int32_t* rows,
                          const int32_t* tile_ad, const LoraPair* table, int layer, int n_layers, int proj, int slot,
                          const float* z, int rmax_p, int ksplits, hipStream_t s) {
  if (n_tiles <= 0 || out <= 0) return hipSuccess;
  if (out % 32 != 0 || slot < 0 || slot > 2 || ksplits < 1) return hipErrorInvalidValue;
  if (kind == 3 && (col0 % 32 != 0 || kd % 32 != 0 || col0 + 2 * kd != out)) return hipErrorInvalidValue;
  lora_up_kernel<<<dim3(n_tiles, (out + 127) / 128), dim3(256), 0, s>>>(dst, ld, out, kind, col0, kd, rows, tile_ad, table,
                                                                       layer, n_layers, proj, slot, z, rmax_p, ksplits);
  return hipGetLastError();
}

hipError_t launch_swiglu_f32(const float* gu, int I, bf16_t* act, int T, hipStream_t s) {
  const int64_t total = (int64_t)T * I;
  if (total <= 0) return hipSuccess;
  swiglu_f32_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s>>>(gu, I, act, total);
  return hipGetLastError();
}
