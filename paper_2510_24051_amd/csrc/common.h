// Shared device/host helpers for the gfx950 kernels: vector types, bf16 conversion, MFMA wrappers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define WAVE 64

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return (float)x; }
// Store that is not meant to stay in the caches.  A kernel's plain stores leave dirty lines behind that are written
// back underneath the next kernel; when that one streams from HBM it pays for them (measured with a stand-alone
// gather of 528 MB: 90 us on its own, 94 / 100 / 108 us right after a kernel that stored 4 / 16 / 64 MiB, and 90 us
// again when the same bytes were stored non-temporally, at no cost to the storing kernel).  Every intermediate here
// is read by a later kernel, which runs on other XCDs with L2s of their own, so nothing is lost by not keeping it.
template <typename T>
__device__ __forceinline__ void store_nt(T* p, T v) {
  __builtin_nontemporal_store(v, p);
}
__device__ __forceinline__ void store_nt(__bf16* p, __bf16 v) {
  __builtin_nontemporal_store(__builtin_bit_cast(uint16_t, v), reinterpret_cast<uint16_t*>(p));
}
// Load of bytes that are read once.  Non-temporal loads are faster on their own (stand-alone measurements: a 528 MB
// gather of 8 KiB blocks 90 -> 80 us, a plain streaming read 5.9 -> 6.45 TB/s) and leave the caches to the data that
// is read again.
template <typename T>
__device__ __forceinline__ T load_nt(const T* p) {
  return __builtin_nontemporal_load(p);
}
__device__ __forceinline__ bf16_t f32_to_bf16(float x) { return (bf16_t)x; }  // v_cvt_pk_bf16_f32: round to nearest even

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// 16-byte views
union Pack16 {
  u32x4 u;
  bf16x8 h;
  uint16_t s[8];
};

// D = A(32x16) * B(16x32) + C.  Lane l carries, for A, row (l % 32) and the 8 contraction
// elements of lane group (l / 32); for B, column (l % 32) and the same 8 contraction elements.
// C/D: lane l carries column (l % 32); register v is row (v / 4) * 8 + (l / 32) * 4 + (v % 4).
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// max(a, b, c) in one instruction.  (fmaxf chains compile to v_max_f32 pairs preceded by a canonicalising
// v_max_f32 x, x per input, because the inputs might be signalling NaNs; MFMA results never are.)
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Exchanges between the two halves of a wave (lane l and l ^ 32) and between neighbouring rows of 16 lanes
// (l and l ^ 16) on the gfx950 swap instructions: v_permlane32_swap with the same register as both operands leaves
// the lower half's value in one result and the upper half's in the other, for every lane; v_permlane16_swap does
// the same for the even and the odd row of each pair of rows.  Plain vector ALU, no trip through the LDS crossbar.
__device__ __forceinline__ float max_xor32(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_xor32(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float max_xor16(float v) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_xor16(float v) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}

// Sum of the eight bf16 values of a packed MFMA operand added to `acc` in fp32 (v_dot2c_f32_bf16 against a pair of
// ones: two values per instruction, the products by 1 are exact).  The softmax normaliser is summed from the
// rounded weights that the PV product multiplies by, so the weights applied and their sum carry the same rounding:
// a row with one visible key returns that key's V row exactly, and with a handful of keys the rounding of the
// weights largely cancels in the final division instead of showing as a 2^-9 relative error of the output.
typedef __bf16 bf16x2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float sum_bf16x8(bf16x8 p, float acc) {
  const bf16x2v ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const bf16x2v pr = {p[2 * i], p[2 * i + 1]};
    acc = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, acc, false);
  }
  return acc;
}

// Tiled weight storage: W[N, K] (Linear layout) is cut into tiles of 32 output rows x 16 inputs,
// 1 KiB each, stored [N/32][K/16]; inside a tile lane l = g * 32 + n holds W[nb*32 + n][kb*16 + g*8 .. +8].
// One 16-byte load per lane is then exactly the B operand of mfma32.
__host__ __device__ __forceinline__ int64_t packed_tile_offset(int nb, int kb, int kblocks) {
  return ((int64_t)nb * kblocks + kb) * 512;  // in bf16 elements
}

// Workgroup barrier without the memory fence of __syncthreads().  The fence makes the compiler wait for every
// outstanding memory operation (s_waitcnt vmcnt(0)) before the barrier, which empties a multi-stage pipeline of
// direct-to-LDS copies at every step.  Callers wait explicitly (s_waitcnt vmcnt(n)) for the copies whose data
// the other waves are about to read; LDS contents are otherwise only written by those copies.
__device__ __forceinline__ void wg_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// s_waitcnt vmcnt(n) as a compiler builtin (not inline asm), so that the compiler's own wait-counter
// bookkeeping knows which copies have landed and does not add a full wait before the next LDS read.
// gfx9 encoding: vmcnt in bits [3:0] and [15:14]; expcnt [6:4] and lgkmcnt [11:8] left at "no wait".
#define PIE_S_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | 0x0F70 | ((((n) >> 4) & 3) << 14))
// s_waitcnt lgkmcnt(0) alone (LDS and scalar-memory operations done; vector-memory loads stay in flight)
#define PIE_S_WAIT_LGKMCNT0() __builtin_amdgcn_s_waitcnt(0xC07F)
