// pie_probe: what this chip delivers for the access patterns the kernels of libpie_mi355 are built on, measured
// with plain loops that do nothing else.  The numbers are the yardsticks the kernel rooflines are discussed against
// (the published peaks are the denominators; these say how much of a peak a pattern can reach at all).
//   1. streaming read of a large buffer (the weight-streaming GEMMs)
//   2. gather of (page, kv head) blocks of 8 KiB in random page order with the decode-attention kernel's load mix
//      (16-byte loads for the K part, 8-byte loads for the V part, next pair in flight)
//   3. re-read of a buffer that fits the last-level cache
//   4. LDS reads per compute unit, 16 and 8 bytes per lane (the operand reads of the tiled GEMM and prefill attention)
//   5. chained bf16 MFMA 32x32x16 on registers (the matrix rate the clock sustains under load)
//   6. the same MFMA loop with independent vector arithmetic (fused multiply-adds, exponentials) issued beside it:
//      how much of the vector work hides under the matrix work (prefill attention's softmax beside its products)
// Standalone program: allocates its own buffers, prints one line per measurement, touches nothing of the library.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <type_traits>
#include <vector>

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define CHECK(x)                                                                   \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) {                                                        \
      printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);        \
      exit(1);                                                                     \
    }                                                                              \
  } while (0)

static hipEvent_t g_e0, g_e1;
template <typename F>
static float best_ms(F&& launch, int reps = 6) {
  float best = 1e30f;
  for (int r = 0; r < reps; ++r) {
    CHECK(hipEventRecord(g_e0));
    launch();
    CHECK(hipEventRecord(g_e1));
    CHECK(hipEventSynchronize(g_e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, g_e0, g_e1));
    if (r) best = std::min(best, ms);  // the first run warms up
  }
  return best;
}

__global__ void fill_kernel(unsigned int* p, size_t n) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    unsigned int x = (unsigned int)i * 2654435761u;
    x ^= x >> 15;
    p[i] = x * 2246822519u;
  }
}

// the same fill with non-temporal stores (the lines are not meant to stay in the caches)
__global__ void fill_nt_kernel(unsigned int* p, size_t n) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    unsigned int x = (unsigned int)i * 2654435761u;
    x ^= x >> 15;
    __builtin_nontemporal_store(x * 2246822519u, p + i);
  }
}

// 1, 3: every thread reads 16 bytes per step, a wave 1 KiB contiguous, eight steps in flight
template <bool NT>
__device__ __forceinline__ u32x4 ld16(const u32x4* p) {
  return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT>
__device__ __forceinline__ u32x2 ld8(const u32x2* p) {
  return NT ? __builtin_nontemporal_load(p) : *p;
}

// the same streaming read with non-temporal loads
__global__ __launch_bounds__(256) void read_nt_kernel(const u32x4* __restrict__ src, size_t n_vec, u32x4* __restrict__ sink) {
  const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
  u32x4 acc = {0, 0, 0, 0};
  size_t i = tid;
  for (; i + 7 * stride < n_vec; i += 8 * stride) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  if (acc.x == 0x12345678 && acc.y == 0x9abcdef0) sink[tid & 1023] = acc;
}

__global__ __launch_bounds__(256) void read_kernel(const u32x4* __restrict__ src, size_t n_vec, u32x4* __restrict__ sink) {
  const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
  u32x4 acc = {0, 0, 0, 0};
  size_t i = tid;
  for (; i + 7 * stride < n_vec; i += 8 * stride) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  if (acc.x == 0x12345678 && acc.y == 0x9abcdef0) sink[tid & 1023] = acc;  // never true: keeps the loads alive
}

// 2: a wave walks `per_wave` pairs of 8 KiB blocks (block = page * 8 + head, a page being 64 KiB): per block four
// 16-byte loads per lane for the first 4 KiB and eight 8-byte loads for the second, the next pair requested before
// the current one is consumed.
template <bool NT = false>
__global__ __launch_bounds__(256, 2) void gather_kernel(const unsigned char* __restrict__ src, const int* __restrict__ blocks,
                                                        int per_wave, int n_waves, u32x4* __restrict__ sink) {
  const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, lane = threadIdx.x & 63;
  if (wave >= n_waves) return;
  const int* bl = blocks + (size_t)wave * per_wave * 2;
  u32x4 acc = {0, 0, 0, 0};
  u32x4 k[2][8];
  u32x2 v[2][16];
  const int voff = 4096 + (((lane >> 5) & 1) * 256 + (lane & 15) * 8 + ((lane >> 4) & 1) * 4) * 2;
  auto fetch = [&](auto sc, int j) {
    constexpr int S = decltype(sc)::value;
    const unsigned char* pa = src + (size_t)bl[2 * j] * 8192;
    const unsigned char* pb = src + (size_t)bl[2 * j + 1] * 8192;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      k[S][i] = ld16<NT>((const u32x4*)(pa + lane * 16 + i * 1024));
      k[S][4 + i] = ld16<NT>((const u32x4*)(pb + lane * 16 + i * 1024));
    }
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const int vo = voff + ((b >> 1) * 512 + (b & 1) * 128) * 2;
      v[S][2 * b] = ld8<NT>((const u32x2*)(pa + vo));
      v[S][2 * b + 1] = ld8<NT>((const u32x2*)(pb + vo));
    }
  };
  auto consume = [&](auto sc) {
    constexpr int S = decltype(sc)::value;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc ^= k[S][i];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      acc.x ^= v[S][i].x;
      acc.y ^= v[S][i].y;
    }
  };
  std::integral_constant<int, 0> s0;
  std::integral_constant<int, 1> s1;
  fetch(s0, 0);
  for (int j = 0; j < per_wave; j += 2) {
    if (j + 1 < per_wave) fetch(s1, j + 1);
    consume(s0);
    if (j + 1 >= per_wave) break;
    if (j + 2 < per_wave) fetch(s0, j + 2);
    consume(s1);
  }
  if (acc.x == 0x12345678 && acc.y == 0x9abcdef0) sink[(wave * 64 + lane) & 1023] = acc;
}

// 4: WAVES waves per compute unit read LDS and nothing else, eight reads in flight per wave (issued back to back, one
// wait for the batch: a loop that waits for every read before it issues the next measures the LDS latency, about a
// quarter of this rate with eight waves).  MODE 0: 16 bytes per lane, 1 KiB contiguous per instruction; 1: 16 bytes
// per lane in the tiled GEMM's swizzled activation layout (rows of 128 bytes, 16-byte chunk c of row r at position
// c ^ ((r >> 1) & 7)); 2: 8 bytes per lane contiguous; 3: rows of 128 bytes without the swizzle.
template <int MODE, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void lds_kernel(unsigned* out, int iters) {
  __shared__ __align__(16) unsigned char lds[65536];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < 65536 / 4; i += WAVES * 64) ((unsigned*)lds)[i] = i;
  __syncthreads();
  unsigned acc = 0;
  int base;
  if (MODE == 0) base = lane * 16;
  else if (MODE == 1) { const int r = lane & 31, g = lane >> 5; base = r * 128 + ((g ^ ((r >> 1) & 7)) << 4); }
  else if (MODE == 2) base = lane * 8;
  else base = (lane & 31) * 128 + (lane >> 5) * 16;
  base += (wave & 7) * 4096;
  unsigned ad[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) ad[u] = (unsigned)(base + (MODE == 1 ? u * 32 : u * 1024)) & 65535u & ~15u;
  for (int it = 0; it < iters; ++it) {
    if (MODE == 2) {
      u32x2 v0, v1, v2, v3, v4, v5, v6, v7;
      asm volatile(
          "ds_read_b64 %0, %8\n ds_read_b64 %1, %9\n ds_read_b64 %2, %10\n ds_read_b64 %3, %11\n"
          "ds_read_b64 %4, %12\n ds_read_b64 %5, %13\n ds_read_b64 %6, %14\n ds_read_b64 %7, %15\n"
          "s_waitcnt lgkmcnt(0)\n"
          : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3), "=&v"(v4), "=&v"(v5), "=&v"(v6), "=&v"(v7)
          : "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3]), "v"(ad[4]), "v"(ad[5]), "v"(ad[6]), "v"(ad[7]));
      acc ^= v0.x ^ v1.x ^ v2.x ^ v3.x ^ v4.x ^ v5.x ^ v6.x ^ v7.x;
    } else {
      u32x4 v0, v1, v2, v3, v4, v5, v6, v7;
      asm volatile(
          "ds_read_b128 %0, %8\n ds_read_b128 %1, %9\n ds_read_b128 %2, %10\n ds_read_b128 %3, %11\n"
          "ds_read_b128 %4, %12\n ds_read_b128 %5, %13\n ds_read_b128 %6, %14\n ds_read_b128 %7, %15\n"
          "s_waitcnt lgkmcnt(0)\n"
          : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3), "=&v"(v4), "=&v"(v5), "=&v"(v6), "=&v"(v7)
          : "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3]), "v"(ad[4]), "v"(ad[5]), "v"(ad[6]), "v"(ad[7]));
      acc ^= v0.x ^ v1.x ^ v2.x ^ v3.x ^ v4.x ^ v5.x ^ v6.x ^ v7.x;
    }
  }
  if (acc == 0x12345) out[tid] = acc;
}

// 5: every wave chains MFMAs on four independent accumulators, operands fixed in registers.  RANDOM: the four MFMAs of
// a round take four different operand pairs of hashed, roughly unit-scale values of both signs, so consecutive MFMAs
// toggle the operand paths the way a contraction over real data does; otherwise one pair of small smooth values.
template <bool RANDOM>
__global__ __launch_bounds__(512) void mfma_kernel(float* out, int iters) {
  bf16x8 a[4], b[4];
  for (int j = 0; j < 4; ++j)
    for (int i = 0; i < 8; ++i) {
      if (RANDOM) {
        unsigned h = (threadIdx.x * 8 + i) * 2654435761u + j * 40503u + blockIdx.x * 97u;
        h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        a[j][i] = (__bf16)(((int)(h & 0xFFFF) - 32768) * (1.0f / 16384.0f));
        b[j][i] = (__bf16)(((int)(h >> 16) - 32768) * (1.0f / 16384.0f));
      } else {
        a[j][i] = (__bf16)(0.001f * (threadIdx.x + i));
        b[j][i] = (__bf16)(0.002f * (threadIdx.x - i));
      }
    }
  f32x16 c[4];
  for (int j = 0; j < 4; ++j)
    for (int v = 0; v < 16; ++v) c[j][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 4; ++j) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[j], c[j], 0, 0, 0);
  }
  float s = 0.f;
  for (int j = 0; j < 4; ++j)
    for (int v = 0; v < 16; ++v) s += c[j][v];
  if (s == 12345.678f) out[threadIdx.x] = s;
}

// 6: sixteen MFMAs on four independent accumulators per iteration and, after them, NV independent vector operations
// on eight registers (fused multiply-adds, or base-2 exponentials).  One or two waves per SIMD.
template <int NV, bool EXP>
__global__ __launch_bounds__(512) void coissue_kernel(float* out, int iters) {
  bf16x8 a, b;
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(0.01f * (threadIdx.x % 7 + i));
    b[i] = (__bf16)(0.02f * (threadIdx.x % 5 + i));
  }
  f32x16 acc[4];
  for (int n = 0; n < 4; ++n)
    for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
  float x[8];
  for (int i = 0; i < 8; ++i) x[i] = 0.001f * (threadIdx.x + i);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < 16; ++m) acc[m % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[m % 4], 0, 0, 0);
#pragma unroll
    for (int j = 0; j < NV; ++j) x[j % 8] = EXP ? __builtin_amdgcn_exp2f(x[j % 8]) : __builtin_fmaf(x[j % 8], 0.999f, 0.001f);
    __builtin_amdgcn_sched_barrier(0);
  }
  float sum = 0;
  for (int n = 0; n < 4; ++n)
    for (int v = 0; v < 16; ++v) sum += acc[n][v];
  for (int i = 0; i < 8; ++i) sum += x[i];
  if (sum == 12345.678f) out[threadIdx.x] = sum;
}

int main() {
  CHECK(hipEventCreate(&g_e0));
  CHECK(hipEventCreate(&g_e1));
  hipDeviceProp_t prop;
  CHECK(hipGetDeviceProperties(&prop, 0));
  const int cus = prop.multiProcessorCount;
  printf("device: %s, %d compute units, clock %.2f GHz (reported maximum)\n", prop.gcnArchName, cus, prop.clockRate / 1e6);

  const size_t big = (size_t)2560 << 20;
  unsigned char* a;
  u32x4* sink;
  CHECK(hipMalloc(&a, big));
  CHECK(hipMalloc(&sink, 1 << 20));
  fill_kernel<<<2048, 256>>>((unsigned int*)a, big / 4);
  CHECK(hipDeviceSynchronize());

  // 1. streaming read, 2 GiB
  {
    const size_t bytes = (size_t)2 << 30;
    float best = 1e30f;
    int best_grid = 0;
    for (int grid : {1024, 2048, 4096, 8192, 16384}) {
      const float ms = best_ms([&] { read_kernel<<<grid, 256>>>((const u32x4*)a, bytes / 16, sink); }, 4);
      if (ms < best) { best = ms; best_grid = grid; }
    }
    printf("streaming read of 2 GiB: %.0f GB/s (%.1f%% of 8000), best grid %d x 256\n", bytes / best / 1e6,
           bytes / best / 1e6 / 80.0, best_grid);
  }
  // 2. page gather, 8064 pages of 64 KiB in random order out of 40960, 8 heads each, 16 pairs per wave
  {
    std::mt19937 rng(1);
    const int n_pages_total = (int)(big / 65536);
    std::vector<int> pages(n_pages_total);
    for (int i = 0; i < n_pages_total; ++i) pages[i] = i;
    std::shuffle(pages.begin(), pages.end(), rng);
    const int used = 8064, per = 16;
    std::vector<int> bl;
    for (int c = 0; c < used / (2 * per); ++c)
      for (int h = 0; h < 8; ++h)
        for (int p = 0; p < 2 * per; ++p) bl.push_back(pages[c * 2 * per + p] * 8 + h);
    const int n_waves = (int)bl.size() / (2 * per);
    int* d;
    CHECK(hipMalloc(&d, bl.size() * 4));
    CHECK(hipMemcpy(d, bl.data(), bl.size() * 4, hipMemcpyHostToDevice));
    const float ms = best_ms([&] { gather_kernel<false><<<(n_waves + 3) / 4, 256>>>(a, d, per, n_waves, sink); });
    const double bytes = (double)bl.size() * 8192;
    printf("gather of %d (page, head) blocks of 8 KiB, %d waves x %d pairs: %.0f GB/s (%.1f%% of 8000), %.1f us for %.1f MB\n",
           (int)bl.size(), n_waves, per, bytes / ms / 1e6, bytes / ms / 1e6 / 80.0, ms * 1e3, bytes / 1e6);
    {
      const float ms_nt = best_ms([&] { gather_kernel<true><<<(n_waves + 3) / 4, 256>>>(a, d, per, n_waves, sink); });
      const float ms_rd = best_ms([&] { read_nt_kernel<<<8192, 256>>>((const u32x4*)a, ((size_t)2 << 30) / 16, sink); }, 4);
      printf("with non-temporal loads: the gather %.1f us, the streaming read of 2 GiB %.0f GB/s\n", ms_nt * 1e3,
             ((double)((size_t)2 << 30)) / ms_rd / 1e6);
    }
    // fixed and marginal cost of the gather: the same number of waves with shorter and longer lists
    {
      printf("gather with non-temporal loads, %d waves, pairs per wave -> time:", n_waves);
      for (int pw : {2, 4, 8, 16}) {
        const float ms = best_ms([&] { gather_kernel<true><<<(n_waves + 3) / 4, 256>>>(a, d, pw, n_waves, sink); });
        printf(" %d: %.1f us (%.0f MB);", pw, ms * 1e3, (double)n_waves * pw * 16384 / 1e6);
      }
      printf("\n");
    }
    // the same gather right after other kernels have streamed 1.5 GiB of other memory (what a serving step does
    // between two decode-attention launches: weights and the LM head), and right after a kernel has written 16 MiB
    {
      unsigned char* other;
      CHECK(hipMalloc(&other, (size_t)1536 << 20));
      fill_kernel<<<2048, 256>>>((unsigned int*)other, ((size_t)1536 << 20) / 4);
      CHECK(hipDeviceSynchronize());
      float best_after_read = 1e30f, sum_after_read = 0.f, best_after_write = 1e30f;
      const int reps = 6;
      for (int r = 0; r < reps; ++r) {
        read_kernel<<<8192, 256>>>((const u32x4*)other, ((size_t)1536 << 20) / 16, sink);
        CHECK(hipEventRecord(g_e0));
        gather_kernel<false><<<(n_waves + 3) / 4, 256>>>(a, d, per, n_waves, sink);
        CHECK(hipEventRecord(g_e1));
        CHECK(hipEventSynchronize(g_e1));
        float t;
        CHECK(hipEventElapsedTime(&t, g_e0, g_e1));
        best_after_read = std::min(best_after_read, t);
        sum_after_read += t;
      }
      printf("the same gather right after a 1.5 GiB read of other memory: %.1f us (best), %.1f us (mean of %d)\n",
             best_after_read * 1e3, sum_after_read / reps * 1e3, reps);
      printf("the same gather right after a kernel that wrote");
      for (size_t kib : {64, 1024, 4096, 16384, 65536}) {
        best_after_write = 1e30f;
        for (int r = 0; r < reps; ++r) {
          fill_kernel<<<(unsigned)std::min<size_t>(2048, kib), 256>>>((unsigned int*)other, (kib << 10) / 4);
          CHECK(hipEventRecord(g_e0));
          gather_kernel<false><<<(n_waves + 3) / 4, 256>>>(a, d, per, n_waves, sink);
          CHECK(hipEventRecord(g_e1));
          CHECK(hipEventSynchronize(g_e1));
          float t;
          CHECK(hipEventElapsedTime(&t, g_e0, g_e1));
          best_after_write = std::min(best_after_write, t);
        }
        printf(" %zu KiB: %.1f us;", kib, best_after_write * 1e3);
      }
      printf(" (best of %d each)\n", reps);
      printf("the same with non-temporal stores in the writing kernel:");
      for (size_t kib : {1024, 4096, 16384, 65536}) {
        best_after_write = 1e30f;
        float best_fill = 1e30f, best_fill_nt = 1e30f;
        for (int r = 0; r < reps; ++r) {
          CHECK(hipEventRecord(g_e1));
          fill_nt_kernel<<<(unsigned)std::min<size_t>(2048, kib), 256>>>((unsigned int*)other, (kib << 10) / 4);
          CHECK(hipEventRecord(g_e0));
          gather_kernel<false><<<(n_waves + 3) / 4, 256>>>(a, d, per, n_waves, sink);
          hipEvent_t e2;
          CHECK(hipEventCreate(&e2));
          CHECK(hipEventRecord(e2));
          CHECK(hipEventSynchronize(e2));
          float t, tf;
          CHECK(hipEventElapsedTime(&t, g_e0, e2));
          CHECK(hipEventElapsedTime(&tf, g_e1, g_e0));
          CHECK(hipEventDestroy(e2));
          best_after_write = std::min(best_after_write, t);
          best_fill_nt = std::min(best_fill_nt, tf);
          CHECK(hipEventRecord(g_e1));
          fill_kernel<<<(unsigned)std::min<size_t>(2048, kib), 256>>>((unsigned int*)other, (kib << 10) / 4);
          CHECK(hipEventRecord(g_e0));
          CHECK(hipEventSynchronize(g_e0));
          CHECK(hipEventElapsedTime(&tf, g_e1, g_e0));
          best_fill = std::min(best_fill, tf);
        }
        printf(" %zu KiB: gather %.1f us (the fill itself %.1f us, with plain stores %.1f us);", kib, best_after_write * 1e3,
               best_fill_nt * 1e3, best_fill * 1e3);
      }
      printf("\n");
      CHECK(hipFree(other));
    }
    CHECK(hipFree(d));
  }
  // 3. re-read of buffers that fit the caches (five passes after one that brings the buffer in)
  for (size_t mb : {32, 128, 256, 1024}) {
    const size_t bytes = mb << 20;
    read_kernel<<<2048, 256>>>((const u32x4*)a, bytes / 16, sink);
    const float ms = best_ms([&] { read_kernel<<<2048, 256>>>((const u32x4*)a, bytes / 16, sink); });
    printf("re-read of %4zu MiB: %.0f GB/s\n", mb, bytes / ms / 1e6);
  }
  // 4. LDS reads
  {
    unsigned* out;
    CHECK(hipMalloc(&out, 1 << 16));
    const int iters = 20000;
    const char* names[4] = {"16 bytes per lane, contiguous", "16 bytes per lane, swizzled 128-byte rows (tiled GEMM operand)",
                            "8 bytes per lane, contiguous", "16 bytes per lane, 128-byte rows without swizzle"};
    for (int waves : {8, 16}) {
      float ms[4];
      if (waves == 8) {
        ms[0] = best_ms([&] { lds_kernel<0, 8><<<cus, 512>>>(out, iters); }, 3);
        ms[1] = best_ms([&] { lds_kernel<1, 8><<<cus, 512>>>(out, iters); }, 3);
        ms[2] = best_ms([&] { lds_kernel<2, 8><<<cus, 512>>>(out, iters); }, 3);
        ms[3] = best_ms([&] { lds_kernel<3, 8><<<cus, 512>>>(out, iters); }, 3);
      } else {
        ms[0] = best_ms([&] { lds_kernel<0, 16><<<cus, 1024>>>(out, iters); }, 3);
        ms[1] = best_ms([&] { lds_kernel<1, 16><<<cus, 1024>>>(out, iters); }, 3);
        ms[2] = best_ms([&] { lds_kernel<2, 16><<<cus, 1024>>>(out, iters); }, 3);
        ms[3] = best_ms([&] { lds_kernel<3, 16><<<cus, 1024>>>(out, iters); }, 3);
      }
      for (int m = 0; m < 4; ++m) {
        const double bytes_cu = (double)iters * 8 * waves * 64 * (m == 2 ? 8 : 16);
        printf("LDS read, %d waves per compute unit, eight reads in flight each, %s: %.1f GB/s per compute unit = %.1f bytes per clock at %.2f GHz\n",
               waves, names[m], bytes_cu / (ms[m] * 1e6), bytes_cu / (ms[m] * 1e6) / (prop.clockRate / 1e6), prop.clockRate / 1e6);
      }
    }
    CHECK(hipFree(out));
  }
  // 5. MFMA on registers: 8 waves per compute unit, 4 chained accumulators each
  {
    float* out;
    CHECK(hipMalloc(&out, 1 << 16));
    const int iters = 200000;
    for (int random = 0; random < 2; ++random) {
      const float ms = random ? best_ms([&] { mfma_kernel<true><<<cus, 512>>>(out, iters); }, 3)
                              : best_ms([&] { mfma_kernel<false><<<cus, 512>>>(out, iters); }, 3);
      const double flops = (double)cus * 8 * iters * 4 * 2.0 * 32 * 32 * 16;
      printf("bf16 MFMA 32x32x16 on registers, %s: %.0f TFLOP/s (%.1f%% of 2500); at 32 cycles per MFMA and SIMD that is a clock of %.2f GHz\n",
             random ? "hashed operands of both signs, four pairs in rotation" : "one pair of small smooth operands",
             flops / ms / 1e9, flops / ms / 1e9 / 25.0, (double)iters * 4 * 2 * 32 / (ms * 1e6));
    }
    CHECK(hipFree(out));
  }
  // 6. MFMA with vector arithmetic beside it
  {
    float* out;
    CHECK(hipMalloc(&out, 1 << 16));
    const int iters = 20000;
    for (int waves : {4, 8}) {
      const dim3 block(waves * 64);
      const float base = best_ms([&] { coissue_kernel<0, false><<<cus, block>>>(out, iters); }, 3);
      struct Case { const char* what; int nv; float ms; } cases[4] = {
          {"64 fused multiply-adds", 64, best_ms([&] { coissue_kernel<64, false><<<cus, block>>>(out, iters); }, 3)},
          {"128 fused multiply-adds", 128, best_ms([&] { coissue_kernel<128, false><<<cus, block>>>(out, iters); }, 3)},
          {"16 exponentials", 16, best_ms([&] { coissue_kernel<16, true><<<cus, block>>>(out, iters); }, 3)},
          {"64 exponentials", 64, best_ms([&] { coissue_kernel<64, true><<<cus, block>>>(out, iters); }, 3)}};
      printf("MFMA + vector work, %d wave(s) per SIMD: 16 MFMAs alone %.1f ns per iteration\n", waves / 4, base * 1e6 / iters);
      for (const Case& c : cases)
        printf("MFMA + vector work, %d wave(s) per SIMD: 16 MFMAs + %s: %.1f ns per iteration, %.2f ns more per vector instruction of the SIMD\n",
               waves / 4, c.what, c.ms * 1e6 / iters, (c.ms - base) * 1e6 / iters / (c.nv * (waves / 4)));
    }
    CHECK(hipFree(out));
  }
  CHECK(hipDeviceSynchronize());
  return 0;
}
