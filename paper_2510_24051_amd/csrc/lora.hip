// LoRA adapters (forward_with_adapter): per-token low-rank updates  y += scale * B (A x)  of the layer's
// projections.  Tokens carry the adapter of their request (-1: none); the pairs of all adapters live in one
// device table indexed [adapter][layer][projection].  Two small kernels per projection group: `lora_down`
// computes z = A x (rank values per token, fp32), `lora_up` adds scale * B z into the projection's output
// (bf16 qkv rows, the fp32 residual stream, or the fp32 gate/up sums in the packed column order of the tiled
// weight).  When gate or up carry an adapter the SwiGLU product cannot be fused into the GEMM epilogue; it is
// taken from the fp32 sums by `swiglu_f32`.
#include "internal.h"

namespace {

// z[t, slot, j] = sum_i x[t, i] * A[j, i]   (j < rank); one workgroup per (token, slot), waves stride over j
__global__ __launch_bounds__(256) void lora_down_kernel(const bf16_t* __restrict__ x, int ldx, int in,
                                                        const int32_t* __restrict__ tok_adapter,
                                                        const LoraPair* __restrict__ table, int layer, int n_layers,
                                                        int proj0, float* __restrict__ z, int rmax) {
  const int t = blockIdx.x, slot = blockIdx.y;
  const int ad = tok_adapter[t];
  if (ad < 0) return;
  const LoraPair p = table[((int64_t)ad * n_layers + layer) * PIE_N_PROJ + proj0 + slot];
  if (p.A == nullptr) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bf16_t* xr = x + (int64_t)t * ldx;
  for (int j = wave; j < p.rank; j += 4) {
    const bf16_t* ar = p.A + (int64_t)j * in;
    float s = 0.f;
    for (int i = lane * 8; i < in; i += 64 * 8) {  // `in` is a multiple of 8
      Pack16 a, b;
      a.u = *reinterpret_cast<const u32x4*>(xr + i);
      b.u = *reinterpret_cast<const u32x4*>(ar + i);
#pragma unroll
      for (int e = 0; e < 8; ++e) s += bf16_bits_to_f32(a.s[e]) * bf16_bits_to_f32(b.s[e]);
    }
    s = wave_sum(s);
    if (lane == 0) z[((int64_t)t * 3 + slot) * rmax + j] = s;
  }
}

// dst[t, column(n)] += scale * sum_j B[n, j] * z[t, slot, j]; one thread per output n
//   kind 0: dst bf16, column = col0 + n       (q, k or v inside the qkv rows)
//   kind 1: dst fp32, column = col0 + n       (residual stream)
//   kind 2: dst fp32, column = (n / 32) * 64 + n % 32 + col0   (gate: col0 = 0, up: col0 = 32; packed order)
__global__ __launch_bounds__(256) void lora_up_kernel(void* __restrict__ dst, int ld, int out, int kind, int col0,
                                                      const int32_t* __restrict__ tok_adapter,
                                                      const LoraPair* __restrict__ table, int layer, int n_layers,
                                                      int proj, int slot, const float* __restrict__ z, int rmax) {
  const int t = blockIdx.x;
  const int n = blockIdx.y * 256 + threadIdx.x;
  const int ad = tok_adapter[t];
  if (ad < 0 || n >= out) return;
  const LoraPair p = table[((int64_t)ad * n_layers + layer) * PIE_N_PROJ + proj];
  if (p.B == nullptr) return;
  const float* zr = z + ((int64_t)t * 3 + slot) * rmax;
  const bf16_t* br = p.B + (int64_t)n * p.rank;
  float s = 0.f;
  for (int j = 0; j < p.rank; ++j) s += bf16_to_f32(br[j]) * zr[j];
  s *= p.scale;
  if (kind == 0) {
    bf16_t* d = reinterpret_cast<bf16_t*>(dst) + (int64_t)t * ld + col0 + n;
    *d = f32_to_bf16(bf16_to_f32(*d) + s);
  } else {
    const int col = kind == 1 ? col0 + n : (n >> 5) * 64 + (n & 31) + col0;
    reinterpret_cast<float*>(dst)[(int64_t)t * ld + col] += s;
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

hipError_t launch_lora_down(const bf16_t* x, int ldx, int in, int T, int n_slots, const int32_t* tok_adapter,
                            const LoraPair* table, int layer, int n_layers, int proj0, float* z, int rmax,
                            hipStream_t s) {
  if (T <= 0 || n_slots <= 0) return hipSuccess;
  lora_down_kernel<<<dim3(T, n_slots), dim3(256), 0, s>>>(x, ldx, in, tok_adapter, table, layer, n_layers, proj0, z, rmax);
  return hipGetLastError();
}

hipError_t launch_lora_up(void* dst, int ld, int out, int kind, int col0, int T, const int32_t* tok_adapter,
                          const LoraPair* table, int layer, int n_layers, int proj, int slot, const float* z, int rmax,
                          hipStream_t s) {
  if (T <= 0 || out <= 0) return hipSuccess;
  lora_up_kernel<<<dim3(T, (out + 255) / 256), dim3(256), 0, s>>>(dst, ld, out, kind, col0, tok_adapter, table, layer,
                                                                 n_layers, proj, slot, z, rmax);
  return hipGetLastError();
}

hipError_t launch_swiglu_f32(const float* gu, int I, bf16_t* act, int T, hipStream_t s) {
  const int64_t total = (int64_t)T * I;
  if (total <= 0) return hipSuccess;
  swiglu_f32_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s>>>(gu, I, act, total);
  return hipGetLastError();
}
