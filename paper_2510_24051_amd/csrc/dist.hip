// Next-token distribution: softmax over the whole vocabulary and exact top-k.
//
// Two kernels so that a handful of rows still fills the chip:
//   topk_chunk : grid (rows, chunks).  A workgroup takes one chunk (<= 8192 logits) of a row, keeps its
//                order-preserving 32-bit keys in registers, reduces the chunk max and sum of exponentials with
//                wavefront reductions, finds the chunk's k-th largest key by radix select and writes the
//                chunk's top-k candidates as 64-bit (key, ~id) composites.
//   topk_merge : grid (rows).  Combines the chunk maxima/sums into the row's softmax normaliser, radix-selects
//                the k largest composites among chunks*k candidates (composites are unique, so ties on the
//                logit resolve to the lower id), sorts those k with a bitonic network and writes ids and
//                probabilities of the full distribution.
//
// Radix select, 8 bits per pass.  Logits share a handful of sign/exponent values, so a histogram of the top
// byte would hammer a few LDS addresses with atomics; instead the top byte is found by walking the byte values
// downward from the maximum's and counting matches in registers (a few steps for any realistic distribution).
// The lower bytes only concern the few keys that share the selected top byte: LDS histogram with atomics.
#include "internal.h"

#define TC_THREADS 512
// keys per thread of the chunk kernel: 16 (chunks of at most 8192 logits) or, when there are enough rows to fill
// the chip with half as many workgroups, 32 (16384 logits): half the block-wide synchronisation per logit
#define TC_LIST 2048  // composites the chunk kernel's short-list selection holds (4 per thread)
#define TM_THREADS 1024
#define TM_PER 16  // composites per thread: at most 16384 candidates per row

__device__ __forceinline__ uint32_t order_key(float z) {
  uint32_t u = __float_as_uint(z);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

// Sum of one unsigned per thread over the workgroup (all threads get the result).  red: [THREADS / 64] words.
template <int THREADS>
__device__ __forceinline__ uint32_t block_sum(uint32_t v, uint32_t* red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  __syncthreads();  // previous use of red is over
  if (lane == 0) red[wave] = v;
  __syncthreads();
  uint32_t t = 0;
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) t += red[w];
  return t;
}

// Top byte of the need-th largest key.  On return *out_b is that byte, *out_need what is still needed among the keys
// that carry it and *out_cnt how many keys carry it (need - *out_need keys have a larger top byte).
// The byte values are walked downward from the maximum's, counting matches in registers: logits of one row share a
// handful of sign/exponent values, so the k-th largest is almost always found within a step or two.  When it is not
// after WALK_STEPS values (a positive maximum over a negative k-th largest lies 128 byte values apart, all the
// exponents of tiny magnitudes in between being empty), the rest of the range is bisected instead: at most eight
// more counts, whatever the distribution.  Every count is uniform over the workgroup, so the control flow is too.
#define WALK_STEPS 4
template <typename KeyT, int PER, int THREADS>
__device__ __forceinline__ void walk_top_byte(const KeyT (&keys)[PER], uint32_t need, int top_byte_max, uint32_t* red,
                                              int* out_b, uint32_t* out_need, uint32_t* out_cnt) {
  constexpr int TOP = sizeof(KeyT) * 8 - 8;
  auto count_in = [&](int lo, int hi) {  // keys whose top byte lies in [lo, hi]
    uint32_t c = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int tb = (int)(keys[i] >> TOP);
      c += (tb >= lo && tb <= hi && keys[i] != 0) ? 1u : 0u;
    }
    return block_sum<THREADS>(c, red);
  };
  int b = top_byte_max;
  uint32_t cnt = 0;
  bool found = false;
  for (int step = 0; step < WALK_STEPS; ++step, --b) {
    cnt = count_in(b, b);
    if (cnt >= need || b == 0) { found = true; break; }
    need -= cnt;
  }
  if (!found) {
    // the answer is the largest byte value t <= hi with count_in(t, hi) >= need (0 when there are fewer keys)
    const int hi = b;
    int lo = 0, up = hi;
    while (lo < up) {
      const int mid = (lo + up + 1) >> 1;
      if (count_in(mid, hi) >= need) lo = mid;
      else up = mid - 1;
    }
    b = lo;
    const uint32_t above = b < hi ? count_in(b + 1, hi) : 0u;
    need -= above;
    cnt = count_in(b, b);
  }
  *out_b = b;
  *out_need = need;
  *out_cnt = cnt;
}

// The lower bytes of the need-th largest among the keys whose top byte is b (eq of them), eight bits per pass with
// an LDS histogram; keys with another top byte take no part.  On return: *out_kth the selected value, *out_need
// how many keys equal to it belong to the top set, *out_eq how many keys equal it in total.  With
// stop_at_shift > 0 the search stops before the passes below that shift when every key sharing the bits decided
// so far is needed anyway (then the low bits of *out_kth are 0 and it is a lower bound of exactly the selected
// set).  hist: 2 x 256 words (the passes alternate between the halves: while the first wave scans one, other
// threads clear the other, so a pass costs two barriers), red: THREADS / 64 words of LDS.
template <typename KeyT, int PER, int THREADS>
__device__ __forceinline__ void select_lower_bytes(const KeyT (&keys)[PER], int b, uint32_t need, uint32_t eq,
                                                   int stop_at_shift, uint32_t* hist, KeyT* sh_prefix,
                                                   uint32_t* sh_need, uint32_t* sh_eq, KeyT* out_kth,
                                                   uint32_t* out_need, uint32_t* out_eq) {
  static_assert(THREADS >= 512, "threads 256..511 clear the idle histogram");
  constexpr int TOP = sizeof(KeyT) * 8 - 8;
  const int tid = threadIdx.x, lane = tid & 63;
  KeyT prefix = (KeyT)b << TOP;
  __syncthreads();  // earlier users of hist and of the shared results are done
  if (tid < 512) hist[tid] = 0u;
  __syncthreads();
  int pass = 0;
  for (int shift = TOP - 8; shift >= 0; shift -= 8, ++pass) {
    if (stop_at_shift > 0 && shift < stop_at_shift && eq == need) break;
    uint32_t* h = hist + (pass & 1) * 256;
    const KeyT hi_mask = ~(KeyT)0 << (shift + 8);
#pragma unroll
    for (int i = 0; i < PER; ++i)
      if ((keys[i] & hi_mask) == prefix && keys[i] != 0) atomicAdd(&h[(uint32_t)(keys[i] >> shift) & 0xFFu], 1u);
    __syncthreads();
    if (tid < 64) {
      // lane L owns bins 255-4L .. 252-4L (descending); a wave scan gives the number of keys in higher bins
      const int b0 = 255 - 4 * lane;
      const uint32_t h0 = h[b0], h1 = h[b0 - 1], h2 = h[b0 - 2], h3 = h[b0 - 3];
      const uint32_t tot = h0 + h1 + h2 + h3;
      uint32_t incl = tot;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
      }
      const uint32_t excl = incl - tot;
      if (excl < need && need <= incl) {
        uint32_t acc = excl, hb = h0;
        int bb = b0;
        if (acc + h0 < need) { acc += h0; bb = b0 - 1; hb = h1;
          if (acc + h1 < need) { acc += h1; bb = b0 - 2; hb = h2;
            if (acc + h2 < need) { acc += h2; bb = b0 - 3; hb = h3; } } }
        *sh_need = need - acc;
        *sh_eq = hb;
        *sh_prefix = prefix | ((KeyT)bb << shift);
      }
    } else if (tid >= 256 && tid < 512) {
      hist[((pass + 1) & 1) * 256 + (tid - 256)] = 0u;  // scanned a pass ago; the next pass counts into it
    }
    __syncthreads();
    need = *sh_need;
    eq = *sh_eq;
    prefix = *sh_prefix;
  }
  *out_kth = prefix;
  *out_need = need;
  *out_eq = eq;
}

// k-th largest of the workgroup's keys (PER per thread in registers, key 0 = padding below every real key):
// the top byte by walking down from `top_byte_max` (the top byte of the largest key), the rest by
// select_lower_bytes.
template <typename KeyT, int PER, int THREADS>
__device__ __forceinline__ void select_kth(const KeyT (&keys)[PER], uint32_t need, int top_byte_max, int stop_at_shift,
                                           uint32_t* hist, uint32_t* red, KeyT* sh_prefix, uint32_t* sh_need,
                                           uint32_t* sh_eq, KeyT* out_kth, uint32_t* out_need, uint32_t* out_eq) {
  int b;
  uint32_t cnt;
  walk_top_byte<KeyT, PER, THREADS>(keys, need, top_byte_max, red, &b, &need, &cnt);
  select_lower_bytes<KeyT, PER, THREADS>(keys, b, need, cnt, stop_at_shift, hist, sh_prefix, sh_need, sh_eq, out_kth,
                                         out_need, out_eq);
}

template <int TC_PER>
__global__ __launch_bounds__(TC_THREADS) void topk_chunk_kernel(const float* __restrict__ logits, int V, int chunk_len,
                                                                int k, float inv_temp,
                                                                unsigned long long* __restrict__ cand,
                                                                float* __restrict__ stats) {
  __shared__ uint32_t hist[512];
  __shared__ uint32_t red[TC_THREADS / 64];
  __shared__ float fred[TC_THREADS / 64];
  __shared__ uint32_t sh_prefix, sh_need, sh_eq, sh_count, sh_count_eq, sh_wave_off[TC_THREADS / 64 + 1];
  __shared__ unsigned long long sh_prefix64;
  __shared__ unsigned long long list[TC_LIST];
  __shared__ float sh_max;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = blockIdx.x, chunk = blockIdx.y, n_chunks = gridDim.y;
  const int start = chunk * chunk_len;
  const int n = min(chunk_len, V - start);
  const float* z = logits + (int64_t)row * V + start;

  // thread t holds logits t*4 + j*(4*THREADS) + e (e < 4, j < PER/4): 16-byte loads, ids recoverable from (j, e)
  uint32_t keys[TC_PER];
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < TC_PER / 4; ++j) {
    const int i = tid * 4 + j * 4 * TC_THREADS;  // start, n and V are multiples of 4
    f32x4 v = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    const bool in = i < n;
    if (in) v = *reinterpret_cast<const f32x4*>(z + i);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      keys[j * 4 + e] = in ? order_key(v[e]) : 0u;
      mx = fmaxf(mx, v[e]);
    }
  }
  mx = wave_max(mx);
  if (lane == 0) fred[wave] = mx;
  __syncthreads();
  if (tid == 0) {
    float m = fred[0];
    for (int w = 1; w < TC_THREADS / 64; ++w) m = fmaxf(m, fred[w]);
    sh_max = m;
    sh_count = 0u;
    sh_count_eq = 0u;
  }
  __syncthreads();
  const float cmax = sh_max;
  // exponentials on the hardware's base-2 instruction (1 ulp): arguments are <= 0, nothing to guard
  const float c2 = inv_temp * 1.44269504088896340736f;
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < TC_PER; ++i)
    if (keys[i] != 0u) sum += __builtin_amdgcn_exp2f((key_to_float(keys[i]) - cmax) * c2);
  sum = wave_sum(sum);
  __syncthreads();
  if (lane == 0) fred[wave] = sum;
  __syncthreads();
  if (tid == 0) {
    float t = 0.f;
    for (int w = 0; w < TC_THREADS / 64; ++w) t += fred[w];
    stats[((int64_t)row * n_chunks + chunk) * 2] = cmax;
    stats[((int64_t)row * n_chunks + chunk) * 2 + 1] = t;
  }
  const int kc = min(k, n);  // candidates this chunk contributes
  unsigned long long* out = cand + ((int64_t)row * n_chunks + chunk) * k;
  auto comp_of = [&](int i) {
    const int id = start + tid * 4 + (i >> 2) * 4 * TC_THREADS + (i & 3);
    return ((unsigned long long)keys[i] << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)id);
  };
  // Usually only a few per cent of the keys share the top byte of the k-th largest or lie above it.  Those are
  // collected as composites in LDS (per-thread counts, a wave scan, one atomic per wave), and the selection runs
  // on that short list, at most TC_LIST / TC_THREADS composites per thread; composites are unique, so equal
  // logits at the cut resolve to the lower ids without a separate pass.  Longer lists (e.g. many equal logits)
  // take the selection over all keys in registers below.
  const int top_byte = (int)(order_key(cmax) >> 24);
  int wb;
  uint32_t w_need, w_cnt;
  walk_top_byte<uint32_t, TC_PER, TC_THREADS>(keys, (uint32_t)kc, top_byte, red, &wb, &w_need, &w_cnt);
  const uint32_t n_list = (uint32_t)kc - w_need + w_cnt;  // keys whose top byte is wb or larger
  if (n_list <= TC_LIST) {
    uint32_t mine = 0u;
#pragma unroll
    for (int i = 0; i < TC_PER; ++i) mine += ((int)(keys[i] >> 24) >= wb && keys[i] != 0u) ? 1u : 0u;
    uint32_t incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t t = __shfl_up(incl, o);
      if (lane >= o) incl += t;
    }
    uint32_t base = 0u;
    if (lane == 63 && incl) base = atomicAdd(&sh_count_eq, incl);  // sh_count_eq: entries of the list so far
    uint32_t pos = __shfl(base, 63) + incl - mine;
#pragma unroll
    for (int i = 0; i < TC_PER; ++i)
      if ((int)(keys[i] >> 24) >= wb && keys[i] != 0u) {
        if (pos < TC_LIST) list[pos] = comp_of(i);
        ++pos;
      }
    __syncthreads();
    unsigned long long c[TC_LIST / TC_THREADS];
#pragma unroll
    for (int j = 0; j < TC_LIST / TC_THREADS; ++j) {
      const uint32_t idx = tid + j * TC_THREADS;
      c[j] = idx < n_list ? list[idx] : 0ull;
    }
    unsigned long long kth64;
    uint32_t need64, eq64;
    // the walk above already found the top byte and what is still needed among the composites that carry it
    select_lower_bytes<unsigned long long, TC_LIST / TC_THREADS, TC_THREADS>(c, wb, w_need, w_cnt, 32, hist, &sh_prefix64,
                                                                             &sh_need, &sh_eq, &kth64, &need64, &eq64);
    // exactly kc composites are >= kth64
#pragma unroll
    for (int j = 0; j < TC_LIST / TC_THREADS; ++j)
      if (c[j] >= kth64 && c[j] != 0ull) {
        const uint32_t p2 = atomicAdd(&sh_count, 1u);
        if (p2 < (uint32_t)kc) out[p2] = c[j];
      }
    for (int i = kc + tid; i < k; i += TC_THREADS) out[i] = 0ull;  // short chunk: pad (a zero never wins)
    return;
  }
  uint32_t kth, need_eq, eq_total;
  select_kth<uint32_t, TC_PER, TC_THREADS>(keys, (uint32_t)kc, (int)(order_key(cmax) >> 24), 0, hist, red, &sh_prefix,
                                           &sh_need, &sh_eq, &kth, &need_eq, &eq_total);
  // keys above kth: any order, slots [need_eq, kc); keys equal to kth: slots [0, need_eq), lowest ids first when
  // only some of them are taken
  const bool split_tie = eq_total != need_eq;
#pragma unroll
  for (int i = 0; i < TC_PER; ++i) {
    if (keys[i] > kth) {
      const uint32_t pos = need_eq + atomicAdd(&sh_count, 1u);
      if (pos < (uint32_t)kc) out[pos] = comp_of(i);  // kc - need_eq keys by construction
    } else if (!split_tie && keys[i] == kth && keys[i] != 0u) {
      const uint32_t pos = atomicAdd(&sh_count_eq, 1u);
      if (pos < need_eq) out[pos] = comp_of(i);
    }
  }
  if (split_tie) {
    // ids ascend with (j, thread, e): walk j outermost; within a j the workgroup's ids are tid*4 + e
    uint32_t eq_seen = 0u;
#pragma unroll  // keys[] must only be indexed by constants, or the array is placed in scratch memory
    for (int j = 0; j < TC_PER / 4; ++j) {
      if (eq_seen >= need_eq) break;  // eq_seen is uniform across the workgroup
      uint32_t mine = 0u;
#pragma unroll
      for (int e = 0; e < 4; ++e) mine += (keys[j * 4 + e] == kth && keys[j * 4 + e] != 0u) ? 1u : 0u;
      uint32_t incl = mine;  // inclusive prefix over the wave, then wave offsets through LDS
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
      }
      __syncthreads();
      if (lane == 63) sh_wave_off[wave + 1] = incl;
      __syncthreads();
      if (tid == 0) {
        sh_wave_off[0] = 0u;
        for (int w = 0; w < TC_THREADS / 64; ++w) sh_wave_off[w + 1] += sh_wave_off[w];
      }
      __syncthreads();
      uint32_t pos = eq_seen + sh_wave_off[wave] + incl - mine;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (keys[j * 4 + e] == kth && keys[j * 4 + e] != 0u) {
          if (pos < need_eq) out[pos] = comp_of(j * 4 + e);
          ++pos;
        }
      eq_seen += sh_wave_off[TC_THREADS / 64];
    }
  }
  for (int i = kc + tid; i < k; i += TC_THREADS) out[i] = 0ull;  // short chunk: pad (a zero never wins)
}

template <int PER>  // composites per thread: the smallest of 2, 4, 8, 16 that holds the row's candidates
__global__ __launch_bounds__(TM_THREADS) void topk_merge_kernel(int n_chunks, int k, float inv_temp,
                                                                const unsigned long long* __restrict__ cand,
                                                                const float* __restrict__ stats, int n2,
                                                                int32_t* __restrict__ out_ids,
                                                                float* __restrict__ out_probs) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  unsigned long long* top = reinterpret_cast<unsigned long long*>(smem_raw);  // [n2 >= k]
  __shared__ uint32_t hist[512];
  __shared__ uint32_t red[TM_THREADS / 64];
  __shared__ unsigned long long sh_prefix;
  __shared__ uint32_t sh_need, sh_eq, sh_count;
  __shared__ uint32_t rank_s[256];
  __shared__ float sh_max, sh_sum;
  const int tid = threadIdx.x;
  const int row = blockIdx.x;
  const int n = n_chunks * k;
  unsigned long long c[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int idx = tid + i * TM_THREADS;
    c[i] = idx < n ? cand[(int64_t)row * n + idx] : 0ull;
  }
  if (tid == 0) {
    float gm = -INFINITY;
    for (int j = 0; j < n_chunks; ++j) gm = fmaxf(gm, stats[((int64_t)row * n_chunks + j) * 2]);
    float s = 0.f;
    for (int j = 0; j < n_chunks; ++j)
      s += stats[((int64_t)row * n_chunks + j) * 2 + 1] * expf((stats[((int64_t)row * n_chunks + j) * 2] - gm) * inv_temp);
    sh_max = gm;
    sh_sum = s;
    sh_count = 0u;
  }
  for (int i = tid; i < n2; i += TM_THREADS) top[i] = 0ull;
  __syncthreads();
  const int top_byte = (int)(order_key(sh_max) >> 24);  // the row maximum is among the candidates
  unsigned long long kth;
  uint32_t need_eq, eq_total;
  // the id half of a composite only matters when equal logits straddle the cut: stop after the key half when
  // every candidate sharing the selected key is needed
  select_kth<unsigned long long, PER, TM_THREADS>(c, (uint32_t)k, top_byte, 32, hist, red, &sh_prefix, &sh_need,
                                                     &sh_eq, &kth, &need_eq, &eq_total);
  // composites are unique: exactly k of them are >= kth
#pragma unroll
  for (int i = 0; i < PER; ++i)
    if (c[i] >= kth && c[i] != 0ull) {
      const uint32_t pos = atomicAdd(&sh_count, 1u);
      if (pos < (uint32_t)n2) top[pos] = c[i];  // exactly k by construction; never write past the buffer
    }
  __syncthreads();
  const float inv_sum = 1.0f / sh_sum, gmax = sh_max;
  auto emit = [&](int slot, unsigned long long v) {
    const int id = (int)(0xFFFFFFFFu - (uint32_t)(v & 0xFFFFFFFFull));
    out_ids[(int64_t)row * k + slot] = id;
    out_probs[(int64_t)row * k + slot] = expf((key_to_float((uint32_t)(v >> 32)) - gmax) * inv_temp) * inv_sum;
  };
  if (n2 <= 256) {
    // Few survivors: every composite finds its place by counting the larger ones (they are unique, so the counts
    // are a permutation).  TM_THREADS / n2 threads share the comparisons of one element; the threads of a wave
    // read the same composite in every step (an LDS broadcast).  Two barriers instead of one per bitonic stage.
    const int parts = TM_THREADS / n2, e = tid & (n2 - 1), part = tid / n2;
    if (tid < n2) rank_s[tid] = 0u;
    __syncthreads();
    if (e < k) {
      const unsigned long long mine = top[e];
      uint32_t larger = 0u;
      for (int j = part; j < k; j += parts) larger += top[j] > mine ? 1u : 0u;
      if (larger) atomicAdd(&rank_s[e], larger);
    }
    __syncthreads();
    if (tid < k) emit((int)rank_s[tid], top[tid]);
    return;
  }
  for (int size = 2; size <= n2; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int i = tid; i < n2 / 2; i += TM_THREADS) {
        const int lo = ((i & ~(stride - 1)) << 1) | (i & (stride - 1));  // stride is a power of two
        const int hi = lo + stride;
        const bool desc = ((lo & size) == 0);
        const unsigned long long a = top[lo], b = top[hi];
        if ((a < b) == desc) {
          top[lo] = b;
          top[hi] = a;
        }
      }
      __syncthreads();
    }
  }
  for (int i = tid; i < k; i += TM_THREADS) emit(i, top[i]);
}

// chunks per row for a vocabulary of V entries; 0 when the combination is not supported
int topk_chunks(int V, int k) {
  int n_chunks = (V + 8191) / 8192;
  if (n_chunks < 1) n_chunks = 1;
  if (n_chunks > 16) return 0;
  return n_chunks;
}

hipError_t launch_topk(const float* logits, int n, int V, int k, float inv_temp, int32_t* out_ids, float* out_probs,
                       unsigned long long* cand_ws, float* stats_ws, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  int n_chunks = topk_chunks(V, k);
  if (n_chunks == 0 || k > 1024 || k > V || k <= 0 || (V & 3)) return hipErrorInvalidValue;
  // with many rows, chunks twice as long still give every CU several workgroups
  const bool wide = n_chunks > 1 && (int64_t)n * n_chunks >= 1024;
  if (wide) n_chunks = (n_chunks + 1) / 2;
  const int per = wide ? 32 : 16;
  int chunk_len = ((V + n_chunks - 1) / n_chunks + 3) / 4 * 4;
  if (chunk_len > TC_THREADS * per || n_chunks * k > TM_THREADS * TM_PER) return hipErrorInvalidValue;
  int n2 = 1;
  while (n2 < k) n2 <<= 1;
  size_t smem_b = (size_t)n2 * 8;
  if (wide)
    topk_chunk_kernel<32><<<dim3(n, n_chunks), dim3(TC_THREADS), 0, s>>>(logits, V, chunk_len, k, inv_temp, cand_ws, stats_ws);
  else
    topk_chunk_kernel<16><<<dim3(n, n_chunks), dim3(TC_THREADS), 0, s>>>(logits, V, chunk_len, k, inv_temp, cand_ws, stats_ws);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int n_cand = n_chunks * k;
  const dim3 mg(n), mb(TM_THREADS);
  if (n_cand <= 2 * TM_THREADS)
    topk_merge_kernel<2><<<mg, mb, smem_b, s>>>(n_chunks, k, inv_temp, cand_ws, stats_ws, n2, out_ids, out_probs);
  else if (n_cand <= 4 * TM_THREADS)
    topk_merge_kernel<4><<<mg, mb, smem_b, s>>>(n_chunks, k, inv_temp, cand_ws, stats_ws, n2, out_ids, out_probs);
  else if (n_cand <= 8 * TM_THREADS)
    topk_merge_kernel<8><<<mg, mb, smem_b, s>>>(n_chunks, k, inv_temp, cand_ws, stats_ws, n2, out_ids, out_probs);
  else
    topk_merge_kernel<TM_PER><<<mg, mb, smem_b, s>>>(n_chunks, k, inv_temp, cand_ws, stats_ws, n2, out_ids, out_probs);
  return hipGetLastError();
}
