// Next-token distribution: softmax over the whole vocabulary and exact top-k.
//
// Two kernels so that a handful of rows still fills the chip:
//   topk_chunk : grid (rows, chunks).  A workgroup stages one chunk of a row's logits in LDS as
//                order-preserving 32-bit keys, reduces the chunk max and sum of exponentials with
//                wavefront reductions, finds the chunk's k-th largest key by radix select (8 bits per
//                pass, LDS histograms, one atomic per distinct bin per wave) and writes the chunk's
//                top-k candidates as 64-bit (key, ~id) composites.
//   topk_merge : grid (rows).  Combines the chunk maxima/sums into the row's softmax normaliser,
//                radix-selects the k largest composites among chunks*k candidates (composites are
//                unique, so ties on the logit resolve to the lower id), sorts them with a bitonic network
//                and writes ids and probabilities of the full distribution.
#include "internal.h"

#define TC_THREADS 512
#define TM_THREADS 1024

__device__ __forceinline__ uint32_t order_key(float z) {
  uint32_t u = __float_as_uint(z);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

// histogram update: one LDS atomic per active lane (the hardware serialises equal addresses within a wave)
__device__ __forceinline__ void hist_add(uint32_t* hist, uint32_t bin, bool active, int lane) {
  if (active) atomicAdd(&hist[bin], 1u);
}

// After the call *sh_prefix holds the `need`-th largest value among the n LDS-resident keys, *sh_need how many
// keys equal to it belong to the top set and *sh_bin_count how many keys equal it in total.  With
// stop_when_unique the passes below `stop_shift` are skipped once every key sharing the prefix found so far
// is needed anyway (then *sh_prefix holds only the decided high bits and is a lower bound of the selected set).
template <typename KeyT, int THREADS>
__device__ __forceinline__ void radix_select(const KeyT* keys, int n, uint32_t need, int top_shift, uint32_t* hist,
                                             KeyT* sh_prefix, uint32_t* sh_need, uint32_t* sh_bin_count,
                                             bool stop_when_unique = false, int stop_shift = 0) {
  const int tid = threadIdx.x, lane = tid & 63;
  if (tid == 0) {
    *sh_prefix = 0;
    *sh_need = need;
  }
  __syncthreads();
  for (int shift = top_shift; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0u;
    __syncthreads();
    const KeyT prefix = *sh_prefix;
    const KeyT hi_mask = (shift == top_shift) ? (KeyT)0 : (~(KeyT)0 << (shift + 8));
    for (int i0 = 0; i0 < n; i0 += THREADS) {
      const int i = i0 + tid;
      KeyT key = i < n ? keys[i] : (KeyT)0;
      const bool act = i < n && (key & hi_mask) == prefix;
      hist_add(hist, (uint32_t)((key >> shift) & 0xFF), act, lane);
    }
    __syncthreads();
    if (tid < 64) {
      // first wave: lane L owns bins 255-4L .. 252-4L (descending); a wave scan gives the number of keys in
      // higher bins, and the one lane whose range crosses `need` picks the bin
      const uint32_t nd = *sh_need;
      const int b0 = 255 - 4 * lane;
      const uint32_t h0 = hist[b0], h1 = hist[b0 - 1], h2 = hist[b0 - 2], h3 = hist[b0 - 3];
      const uint32_t tot = h0 + h1 + h2 + h3;
      uint32_t incl = tot;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
      }
      const uint32_t excl = incl - tot;
      if (excl < nd && nd <= incl) {
        uint32_t acc = excl;
        int b = b0;
        if (acc + h0 < nd) { acc += h0; b = b0 - 1;
          if (acc + h1 < nd) { acc += h1; b = b0 - 2;
            if (acc + h2 < nd) { acc += h2; b = b0 - 3; } } }
        *sh_need = nd - acc;
        *sh_prefix = prefix | ((KeyT)b << shift);
        *sh_bin_count = (b == b0) ? h0 : (b == b0 - 1) ? h1 : (b == b0 - 2) ? h2 : h3;
      }
    }
    __syncthreads();
    if (stop_when_unique && *sh_bin_count == *sh_need && shift <= stop_shift) break;  // uniform: shared values
  }
}

__global__ __launch_bounds__(TC_THREADS) void topk_chunk_kernel(const float* __restrict__ logits, int V, int chunk_len,
                                                                int k, float inv_temp,
                                                                unsigned long long* __restrict__ cand,
                                                                float* __restrict__ stats) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  uint32_t* keys = reinterpret_cast<uint32_t*>(smem_raw);  // [chunk_len]
  __shared__ float red[TC_THREADS / 64];
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sh_prefix, sh_need, sh_bin, sh_count, sh_count_eq, sh_wave_off[TC_THREADS / 64 + 1];
  __shared__ float sh_max;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = blockIdx.x, chunk = blockIdx.y, n_chunks = gridDim.y;
  const int start = chunk * chunk_len;
  const int n = min(chunk_len, V - start);
  const float* z = logits + (int64_t)row * V + start;

  float mx = -INFINITY;
  for (int i = tid * 4; i < n; i += TC_THREADS * 4) {  // start and V are multiples of 4
    f32x4 v = *reinterpret_cast<const f32x4*>(z + i);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      keys[i + e] = order_key(v[e]);
      mx = fmaxf(mx, v[e]);
    }
  }
  mx = wave_max(mx);
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  if (tid == 0) {
    float m = red[0];
    for (int w = 1; w < TC_THREADS / 64; ++w) m = fmaxf(m, red[w]);
    sh_max = m;
  }
  __syncthreads();
  const float cmax = sh_max;
  float sum = 0.f;
  for (int i = tid; i < n; i += TC_THREADS) sum += expf((key_to_float(keys[i]) - cmax) * inv_temp);
  sum = wave_sum(sum);
  __syncthreads();
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  if (tid == 0) {
    float t = 0.f;
    for (int w = 0; w < TC_THREADS / 64; ++w) t += red[w];
    stats[((int64_t)row * n_chunks + chunk) * 2] = cmax;
    stats[((int64_t)row * n_chunks + chunk) * 2 + 1] = t;
    sh_count = 0u;
    sh_count_eq = 0u;
  }
  const int kc = min(k, n);  // candidates this chunk contributes
  radix_select<uint32_t, TC_THREADS>(keys, n, (uint32_t)kc, 24, hist, &sh_prefix, &sh_need, &sh_bin);
  const uint32_t kth = sh_prefix, need_eq = sh_need;
  const bool split_tie = sh_bin != need_eq;  // some but not all keys equal to kth are taken: lowest ids win
  unsigned long long* out = cand + ((int64_t)row * n_chunks + chunk) * k;
  // keys above kth: any order, slots [need_eq, kc); keys equal to kth: lowest ids first, slots [0, need_eq)
  uint32_t eq_seen = 0u;
  for (int base = 0; base < n; base += TC_THREADS) {
    const int i = base + tid;
    uint32_t key = 0u;
    bool gt = false, eq = false;
    if (i < n) {
      key = keys[i];
      gt = key > kth;
      eq = key == kth;
    }
    const unsigned long long comp = ((unsigned long long)key << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)(start + i));
    if (gt) out[need_eq + atomicAdd(&sh_count, 1u)] = comp;
    if (!split_tie) {
      if (eq) out[atomicAdd(&sh_count_eq, 1u)] = comp;
    } else if (eq_seen < need_eq) {  // uniform across the workgroup
      const unsigned long long bal = __ballot(eq);
      const uint32_t before = (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
      if (lane == 0) sh_wave_off[wave + 1] = (uint32_t)__popcll(bal);
      __syncthreads();
      if (tid == 0) {
        sh_wave_off[0] = 0u;
        for (int w = 0; w < TC_THREADS / 64; ++w) sh_wave_off[w + 1] += sh_wave_off[w];
      }
      __syncthreads();
      const uint32_t pos = eq_seen + sh_wave_off[wave] + before;
      if (eq && pos < need_eq) out[pos] = comp;
      eq_seen += sh_wave_off[TC_THREADS / 64];
      __syncthreads();
    }
  }
  for (int i = kc + tid; i < k; i += TC_THREADS) out[i] = 0ull;  // short chunk: pad (a zero never wins)
}

__global__ __launch_bounds__(TM_THREADS) void topk_merge_kernel(const float* __restrict__ logits, int V, int n_chunks,
                                                                int k, float inv_temp,
                                                                const unsigned long long* __restrict__ cand,
                                                                const float* __restrict__ stats, int n2,
                                                                int32_t* __restrict__ out_ids,
                                                                float* __restrict__ out_probs) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  unsigned long long* c = reinterpret_cast<unsigned long long*>(smem_raw);  // [n2 >= n_chunks * k]
  __shared__ float sh_max, sh_sum;
  const int tid = threadIdx.x;
  const int row = blockIdx.x;
  const int n = n_chunks * k;
  for (int i = tid; i < n; i += TM_THREADS) c[i] = cand[(int64_t)row * n + i];
  if (tid == 0) {
    float gm = -INFINITY;
    for (int j = 0; j < n_chunks; ++j) gm = fmaxf(gm, stats[((int64_t)row * n_chunks + j) * 2]);
    float s = 0.f;
    for (int j = 0; j < n_chunks; ++j)
      s += stats[((int64_t)row * n_chunks + j) * 2 + 1] * expf((stats[((int64_t)row * n_chunks + j) * 2] - gm) * inv_temp);
    sh_max = gm;
    sh_sum = s;
  }
  __syncthreads();
  // composites are unique and order by (logit, then lower id): a descending bitonic sort of all candidates
  // puts the row's top-k first
  unsigned long long* top = c;
  for (int i = n + tid; i < n2; i += TM_THREADS) c[i] = 0ull;
  __syncthreads();
  for (int size = 2; size <= n2; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int i = tid; i < n2 / 2; i += TM_THREADS) {
        const int lo = ((i & ~(stride - 1)) << 1) | (i & (stride - 1));  // stride is a power of two
        const int hi = lo + stride;
        const bool desc = ((lo & size) == 0);
        const unsigned long long a = c[lo], b = c[hi];
        if ((a < b) == desc) {
          c[lo] = b;
          c[hi] = a;
        }
      }
      __syncthreads();
    }
  }
  const float inv_sum = 1.0f / sh_sum, gmax = sh_max;
  for (int i = tid; i < k; i += TM_THREADS) {
    const unsigned long long v = top[i];
    const int id = (int)(0xFFFFFFFFu - (uint32_t)(v & 0xFFFFFFFFull));
    out_ids[(int64_t)row * k + i] = id;
    out_probs[(int64_t)row * k + i] = expf((key_to_float((uint32_t)(v >> 32)) - gmax) * inv_temp) * inv_sum;
  }
}

// chunks per row for a vocabulary of V entries and top-k k; 0 when the combination is not supported
int topk_chunks(int V, int k) {
  int n_chunks = (V + 8191) / 8192;
  if (n_chunks < 1) n_chunks = 1;
  if (n_chunks > 16) return 0;
  return n_chunks;
}

hipError_t launch_topk(const float* logits, int n, int V, int k, float inv_temp, int32_t* out_ids, float* out_probs,
                       unsigned long long* cand_ws, float* stats_ws, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const int n_chunks = topk_chunks(V, k);
  if (n_chunks == 0 || k > 1024 || k > V || k <= 0 || (V & 3)) return hipErrorInvalidValue;
  int chunk_len = ((V + n_chunks - 1) / n_chunks + 3) / 4 * 4;
  size_t smem_a = (size_t)chunk_len * 4;
  int n2 = 1;
  while (n2 < n_chunks * k) n2 <<= 1;
  size_t smem_b = (size_t)n2 * 8;
  hipError_t e = hipFuncSetAttribute((const void*)topk_merge_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_b);
  if (e != hipSuccess) return e;
  topk_chunk_kernel<<<dim3(n, n_chunks), dim3(TC_THREADS), smem_a, s>>>(logits, V, chunk_len, k, inv_temp, cand_ws,
                                                                       stats_ws);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  topk_merge_kernel<<<dim3(n), dim3(TM_THREADS), smem_b, s>>>(logits, V, n_chunks, k, inv_temp, cand_ws, stats_ws, n2,
                                                               out_ids, out_probs);
  return hipGetLastError();
}
