// Next-token distribution: softmax over the whole vocabulary and exact top-k, one workgroup per row.
//
// Steps: (1) row max and sum of exp((z - max)/T) with wavefront reductions; (2) exact radix select of the
// k-th largest logit on an order-preserving 32-bit key, 8 bits per pass, LDS histograms; (3) gather: every
// key above the threshold, and the lowest-id keys equal to it until k are found (ordered block scan);
// (4) bitonic sort of the k candidates by (logit descending, id ascending); (5) write ids and
// probabilities of the full distribution.
#include "internal.h"

#define TK_THREADS 1024
#define TK_MAXK 1024

__device__ __forceinline__ uint32_t order_key(float z) {
  uint32_t u = __float_as_uint(z);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(TK_THREADS) void topk_kernel(const float* __restrict__ logits, int V, int k,
                                                          float inv_temp, int32_t* __restrict__ out_ids,
                                                          float* __restrict__ out_probs) {
  __shared__ float red[TK_THREADS / 64];
  __shared__ uint32_t hist[256];
  __shared__ unsigned long long cand[TK_MAXK];
  __shared__ uint32_t sh_prefix, sh_need, sh_count, sh_wave_off[TK_THREADS / 64 + 1];
  __shared__ float sh_max, sh_sum;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* z = logits + (int64_t)blockIdx.x * V;

  // (1) max, then sum of exponentials
  float mx = -INFINITY;
  for (int i = tid; i < V; i += TK_THREADS) mx = fmaxf(mx, z[i]);
  mx = wave_max(mx);
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  if (tid == 0) {
    float m = red[0];
    for (int w = 1; w < TK_THREADS / 64; ++w) m = fmaxf(m, red[w]);
    sh_max = m;
  }
  __syncthreads();
  const float zmax = sh_max;
  float sum = 0.f;
  for (int i = tid; i < V; i += TK_THREADS) sum += expf((z[i] - zmax) * inv_temp);
  sum = wave_sum(sum);
  __syncthreads();
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  if (tid == 0) {
    float t = 0.f;
    for (int w = 0; w < TK_THREADS / 64; ++w) t += red[w];
    sh_sum = t;
    sh_prefix = 0u;
    sh_need = (uint32_t)k;
  }
  __syncthreads();

  // (2) radix select: after the pass over byte b, sh_prefix holds the top (32 - 8b) bits of the k-th largest key
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (tid < 256) hist[tid] = 0u;
    __syncthreads();
    const uint32_t prefix = sh_prefix;
    const uint32_t hi_mask = (shift == 24) ? 0u : (0xFFFFFFFFu << (shift + 8));
    for (int i = tid; i < V; i += TK_THREADS) {
      uint32_t key = order_key(z[i]);
      if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 0xFFu], 1u);
    }
    __syncthreads();
    if (tid == 0) {
      uint32_t need = sh_need, acc = 0u;
      int b = 255;
      for (; b > 0; --b) {
        if (acc + hist[b] >= need) break;
        acc += hist[b];
      }
      sh_need = need - acc;  // still needed among keys whose byte equals b
      sh_prefix = prefix | ((uint32_t)b << shift);
    }
    __syncthreads();
  }
  const uint32_t kth = sh_prefix;    // key of the k-th largest logit
  const uint32_t need_eq = sh_need;  // how many keys equal to kth belong to the top-k
  if (tid == 0) sh_count = 0u;
  __syncthreads();

  // (3) gather.  Keys above kth go to slots [need_eq, k) in any order; keys equal to kth fill slots
  // [0, need_eq) in ascending id order.
  uint32_t eq_seen = 0u;
  for (int base = 0; base < V; base += TK_THREADS) {
    const int i = base + tid;
    uint32_t key = 0u;
    bool gt = false, eq = false;
    if (i < V) {
      key = order_key(z[i]);
      gt = key > kth;
      eq = key == kth;
    }
    if (gt) {
      uint32_t slot = need_eq + atomicAdd(&sh_count, 1u);
      cand[slot] = ((unsigned long long)key << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)i);
    }
    if (eq_seen < need_eq) {  // uniform across the block
      const unsigned long long bal = __ballot(eq);
      const uint32_t before = __popcll(bal & ((1ull << lane) - 1ull));
      if (lane == 0) sh_wave_off[wave + 1] = __popcll(bal);
      __syncthreads();
      if (tid == 0) {
        sh_wave_off[0] = 0u;
        for (int w = 0; w < TK_THREADS / 64; ++w) sh_wave_off[w + 1] += sh_wave_off[w];
      }
      __syncthreads();
      const uint32_t pos = eq_seen + sh_wave_off[wave] + before;
      if (eq && pos < need_eq) cand[pos] = ((unsigned long long)key << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)i);
      eq_seen += sh_wave_off[TK_THREADS / 64];
      __syncthreads();
    }
  }
  __syncthreads();

  // (4) bitonic sort, descending on (key, ~id): larger logit first, then smaller id
  int n2 = 1;
  while (n2 < k) n2 <<= 1;
  for (int i = k + tid; i < n2; i += TK_THREADS) cand[i] = 0ull;
  __syncthreads();
  for (int size = 2; size <= n2; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int i = tid; i < n2 / 2; i += TK_THREADS) {
        int lo = ((i / stride) * stride * 2) + (i % stride);
        int hi = lo + stride;
        bool desc = ((lo & size) == 0);
        unsigned long long a = cand[lo], b = cand[hi];
        if ((a < b) == desc) {
          cand[lo] = b;
          cand[hi] = a;
        }
      }
      __syncthreads();
    }
  }

  // (5) output
  const float inv_sum = 1.0f / sh_sum;
  for (int i = tid; i < k; i += TK_THREADS) {
    unsigned long long c = cand[i];
    int id = (int)(0xFFFFFFFFu - (uint32_t)(c & 0xFFFFFFFFull));
    out_ids[(int64_t)blockIdx.x * k + i] = id;
    out_probs[(int64_t)blockIdx.x * k + i] = expf((z[id] - zmax) * inv_temp) * inv_sum;
  }
}

hipError_t launch_topk(const float* logits, int n, int V, int k, float inv_temp, int32_t* out_ids, float* out_probs,
                       hipStream_t s) {
  if (n <= 0) return hipSuccess;
  if (k > TK_MAXK || k > V || k <= 0) return hipErrorInvalidValue;
  topk_kernel<<<dim3(n), dim3(TK_THREADS), 0, s>>>(logits, V, k, inv_temp, out_ids, out_probs);
  return hipGetLastError();
}
