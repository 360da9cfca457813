// Internal structures and kernel launchers shared by the translation units of libpie_mi355.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <utility>
#include <vector>

#include "../../include/pie_mi355.h"
#include "common.h"

#define PAGE 16  // tokens per block of the KvPage pool the kernels are built for (a KvPage is one or two blocks)

// ---- tiled weights ---------------------------------------------------------------------------
struct PackedWeight {
  bf16_t* data = nullptr;
  int N = 0;   // logical output rows
  int K = 0;   // inputs (multiple of 16)
  int NB = 0;  // number of 32-row blocks stored (N rounded up)
};

struct LayerWeights {
  bool loaded = false;
  bf16_t* g1 = nullptr;
  bf16_t* g2 = nullptr;
  PackedWeight wqkv, wo, wgu, wdown;  // wgu: gate/up interleaved in 32-row blocks
};

// ---- KvPage pool layout ----------------------------------------------------------------------
// pool[layer][page][kv_head] is one block of 2 * PAGE * D bf16: a K part then a V part, both arranged
// so that one 16-byte load per lane is an mfma32 A operand.
//   K(token t, d): (d/16)*256 + ((d%16)/8)*128 + swap23(t)*8 + d%8      swap23 exchanges bits 2 and 3 of t
//   V(token t, d): PAGE*D + (d/32)*512 + (t/8)*256 + (d%32)*8 + t%8
__host__ __device__ __forceinline__ int swap23(int t) { return (t & 3) | ((t & 4) << 1) | ((t & 8) >> 1); }
__host__ __device__ __forceinline__ int k_elem_offset(int t, int d) {
  return (d >> 4) * 256 + ((d >> 3) & 1) * 128 + swap23(t) * 8 + (d & 7);
}
__host__ __device__ __forceinline__ int v_elem_offset(int t, int d, int D) {
  return PAGE * D + (d >> 5) * 512 + (t >> 3) * 256 + (d & 31) * 8 + (t & 7);
}

// ---- LoRA adapters ---------------------------------------------------------------------------
struct LoraPair {  // one projection of one layer of one adapter; device copies owned by the context
  bf16_t* A = nullptr;  // [rank_p, in], rows past the rank are zero
  bf16_t* B = nullptr;  // [out, rank_p], columns past the rank are zero
  int32_t rank = 0;
  int32_t rank_p = 0;   // rank rounded up to a multiple of 16 (one MFMA contraction step)
  float scale = 0.f;
};

// ---- batch plan ------------------------------------------------------------------------------
struct ReqInfo {       // one per request, device + host
  int32_t tok0;        // first token
  int32_t n_new;       // new tokens
  int32_t kv_len;      // after append
  int32_t visit0;      // first entry of this request's visit list
  int32_t n_visit;     // pages with at least one visible key, logical order
  int32_t wpr;         // mask words per row (0: inferred causal)
  int64_t mask_off;    // word offset of the request's first row
  int32_t dec_index;   // index among the decode-path requests, or -1
  int32_t pair0;       // prefill path: first entry of the request's list of visited page pairs
};

struct DecodeCol {     // one query column of a column group: (request token, head within the kv group)
  int32_t tok;         // token index (row of q), -1 = unused column
  int32_t hg;          // head within the group
  int32_t kv_len;      // of the column's request
  int32_t lim;         // last logical index visible under the causal rule: kv_len - n_new + i
  int32_t wpr;         // mask words per row, 0 = inferred causal
  int32_t pad;
  int64_t mask_row;    // word offset of this token's mask row
};
// A column group is a set of up to 16 query columns that walk the same pages: the rows of one decode-path
// request, or of several requests whose page tables name the same physical page at the same logical index
// (shared prefixes), so that each K/V block is read once for all of them.
struct DecodeSeg { int32_t cgroup, hk, n_pairs, pad; };  // a run of page pairs of one (column group, kv head) inside one wave's share
struct DecodeWave { int32_t seg0, n_seg, n_pairs, pad; };  // a wave's share: segments [seg0, seg0 + n_seg)
struct PrefillItem { int32_t r, qb, hk, pad; };  // query block qb (32 tokens) of request r for kv head hk; r < 0: empty slot

struct pie_batch {
  const pie_ctx* owner = nullptr;  // the context that deserialised the batch: its pools, ranges and wave count are baked in
  int32_t R = 0, T = 0;
  std::vector<int32_t> out_ids_host;  // host copy of the output Embed ids (pie_forward_dist)
  void* dev_blob = nullptr;  // single allocation holding every array below
  size_t dev_blob_bytes = 0;
  float* rope_angles = nullptr;  // [T, D] cos | sin of every token's rotary angles (made once per batch on the GPU)
  int32_t *in_ids = nullptr, *out_ids = nullptr, *pos = nullptr, *tok_page = nullptr, *tok_slot = nullptr;
  // tokens of requests that name an adapter, grouped by adapter in tiles of 32 rows (null / 0: no adapters)
  int32_t* lora_rows = nullptr;        // [n_lora_tiles * 32] token index, -1 = padding
  int32_t* lora_tile_ad = nullptr;     // [n_lora_tiles] adapter of the tile
  int n_lora_tiles = 0;
  std::vector<int32_t> used_adapters;  // host: distinct adapters named by the batch
  int32_t *visit_phys = nullptr, *visit_logical = nullptr;
  int32_t* visit_pairs = nullptr;  // prefill-path requests: (physical, logical, physical, logical) per pair of visited pages
  uint32_t* mask_words = nullptr;
  ReqInfo* reqs = nullptr;
  DecodeSeg* dsegs = nullptr;
  DecodeWave* dwaves = nullptr;  // [n_dwaves]
  int2* wave_pg = nullptr;       // [n_dwaves, dslots] (page * Hkv + kv head, logical page) of every pair slot
  DecodeCol* dcols = nullptr;      // [n_cgroups, 16]
  int32_t* mref_indptr = nullptr;  // [n_dec_reqs * Hkv + 1] partial rows to merge per (decode request, kv head)
  int32_t* mrefs = nullptr;        // first partial row (segment * rows_cap + first column of the request)
  PrefillItem* pitems = nullptr;
  int32_t* dec_reqs = nullptr;  // request indices on the decode path
  int32_t n_dsegs = 0, n_dwaves = 0, dslots = 0, n_pitems = 0, n_dec_reqs = 0, rows_cap = 0;
  std::vector<PrefillItem> pwork_host;  // host copy of the prefill launch layout (inspection)
  // workgroups of the two prefill launches, (query block, kv head) items laid out per XCD and padded: the first
  // n_pwork entries of pitems run with plain bf16 softmax weights, the following n_pwork_lo (query blocks whose rows
  // may see few keys: bitmap masks, causal blocks that start within the first 64 keys) with weights as bf16 pairs
  int32_t n_pwork = 0, n_pwork_lo = 0;
  float* part_o = nullptr;   // [n_dsegs * rows_cap, D]
  float* part_ml = nullptr;  // [n_dsegs * rows_cap, 2]
  int64_t work[6] = {0, 0, 0, 0, 0, 0};
};

struct pie_ctx {
  pie_model_desc m;
  pie_pool_desc p;
  hipStream_t stream = nullptr;
  int device = 0;
  int wave_slots = 2048;  // waves the chip keeps resident for the decode-attention kernel
  int blocks_per_page = 1;  // a KvPage is this many consecutive 16-token blocks of the pool (page_size / 16)
  bool host_only = false; // pie_create_planner: deserialises and plans batches, owns nothing on a device
  bf16_t* embeds = nullptr;
  bf16_t* kv = nullptr;
  size_t kv_layer_elems = 0;
  std::vector<LayerWeights> layers;
  bool head_loaded = false;
  bf16_t* g_final = nullptr;
  PackedWeight wlm;
  double* inv_freq = nullptr;
  bf16_t* table = nullptr;             // embedding table [vocab, H] (embed_txt)
  std::vector<int32_t> embed_pos;      // host: sequence position recorded with each Embed by embed_txt, -1 = none
  std::vector<uint16_t> page_mask;     // host: token-level visibility bits of every KvPage (mask_kvpage), all layers
  std::vector<LoraPair> lora;          // host mirror of the adapter table [max_adapters][n_layers][PIE_N_PROJ]
  LoraPair* lora_dev = nullptr;        // the same table on the device
  float* lora_z = nullptr;             // [lora_z_rows, 3, padded max rank] fp32: A x of up to three projections sharing an input
  size_t lora_z_rows = 0;
  float* gu32 = nullptr;               // [T, 2 I] fp32 gate/up sums (packed column order) for adapted gate/up
  float* x32 = nullptr;                // [T, H] wide layer input of the layers after the first (n_layers > 1)
  // workspace
  bf16_t *xn = nullptr, *qkv = nullptr, *attn = nullptr, *act = nullptr, *en = nullptr;
  float *h = nullptr, *splitk = nullptr, *logits = nullptr, *topk_stats = nullptr;
  unsigned long long* topk_cand = nullptr;
  size_t splitk_elems = 0;
  // device blocks of destroyed batches, kept for the next pie_batch_create (a serving loop creates and destroys a
  // batch per step; hipMalloc + hipFree cost more than the deserialisation itself)
  std::vector<std::pair<void*, size_t>> blob_pool;
  // host image of a batch's device block, reused from batch to batch (pinned when the context has a device, so
  // the copy to the device is a single DMA; plain memory on planner contexts)
  unsigned char* host_blob = nullptr;
  size_t host_blob_cap = 0;
  bool host_blob_pinned = false;
  std::vector<uint32_t> page_stamp;  // host: per pool page, the last batch plan that counted it (distinct-page statistic)
  uint32_t page_stamp_id = 0;
  int32_t* ids_dev = nullptr;  // staging for id lists of the small resource calls
  size_t ids_cap = 0;
  int last_T = 0, last_dist_n = 0;
  const float* last_logits = nullptr;  // logits of the last get_next_dist call (workspace or static scratch)
  unsigned char* static_scratch = nullptr;  // device address of this GPU's static scratch array (pie_get_next_dist_static)
  // timing
  bool timing = false;
  hipEvent_t ev[2 * PIE_N_STAGES];
  bool ev_used[PIE_N_STAGES];
  char err[512];
};

// ---- launchers (all enqueue on `s`, return hipGetLastError) ------------------------------------
hipError_t launch_pack_weight(const bf16_t* s0, int r0, const bf16_t* s1, int r1, const bf16_t* s2, int r2, int K,
                              int interleave, bf16_t* dst, int NB, hipStream_t s);
hipError_t launch_rmsnorm_embed(const bf16_t* embeds, const int32_t* ids, const bf16_t* gain, bf16_t* out, int rows,
                                int H, float eps, hipStream_t s);
hipError_t launch_rmsnorm_f32(const float* x, const bf16_t* gain, bf16_t* out, int rows, int H, float eps,
                              hipStream_t s);
// part/splits: when splits > 0 the q, k, v values are not read from qkv but summed from the split-K partials
// [split][T][NP] of the QKV product (then rounded to bf16 as the epilogue would have stored them).
hipError_t launch_rope_append(bf16_t* qkv, int T, int Hq, int Hkv, int D, const int32_t* pos, const int32_t* tok_page,
                              const int32_t* tok_slot, const float* angles, bf16_t* kv_layer, const float* part,
                              int splits, int NP, hipStream_t s);
// angles [T, D]: cos (first D/2) and sin (last D/2) of pos[t] * inv_freq[i], double precision rounded to float
hipError_t launch_rope_table(const int32_t* pos, const double* inv_freq, int T, int D, float* angles, hipStream_t s);
// Split-K epilogue of a residual projection fused with the RMSNorm that follows it: wide[m] = residual[m] + sum of
// the partials [split][rows][NP] (residual: resid fp32 [rows, H], or Embed ids[m] when resid is null), and
// out[m] = bf16(rmsnorm(wide[m]) * gain).
hipError_t launch_splitk_resid_norm(const float* part, int splits, int NP, const float* resid, const bf16_t* embeds,
                                    const int32_t* ids, float* wide, const bf16_t* gain, bf16_t* out, int rows, int H,
                                    float eps, hipStream_t s);
hipError_t launch_embed_copy(bf16_t* embeds, const int32_t* ids, int n, int H, bf16_t* buf, int to_pool,
                             hipStream_t s);
hipError_t launch_kv_token_copy(bf16_t* kv, size_t layer_elems, int n_layers, const int32_t* src_pages,
                                const int32_t* src_slots, const int32_t* dst_pages, const int32_t* dst_slots, int n,
                                int Hkv, int D, hipStream_t s);
hipError_t launch_embed_gather(bf16_t* embeds, const int32_t* ids, const int32_t* tok, int n, int H,
                               const bf16_t* table, hipStream_t s);
hipError_t launch_kv_copy(bf16_t* kv_layer, const int32_t* pages, const int32_t* slots, int n, int Hkv, int D,
                          bf16_t* k, bf16_t* v, int to_pool, hipStream_t s);

enum EpiMode {
  EPI_STORE_BF16 = 0,    // out bf16 [M, N]
  EPI_RESID_EMBED = 1,   // out fp32 [M, N] = embeds[in_ids[m]][n] + acc, or resid[m][n] + acc when resid is given
  EPI_SWIGLU = 2,        // out bf16 [M, N/2] = silu(gate) * up, gate/up interleaved in 32-column blocks
  EPI_RESID_OUT = 3,     // embeds[out_ids[m]][n] = bf16(resid[m][n] + acc) when out_ids[m] >= 0, or, when out is
                         // given, out fp32 [M, N] = resid[m][n] + acc for every row
  EPI_STORE_F32 = 4      // out fp32 [M, N]
};
struct EpiArgs {
  int mode;
  void* out;
  int ldo;
  bf16_t* embeds;
  const int32_t* ids;
  const float* resid;
  int H;
};
// C[M, N] = A[M, K] (bf16 row-major, leading dimension lda) x W^T with the epilogue above.
// deferred_splits (optional): when the product was split along K, the epilogue kernel is not launched and
// *deferred_splits receives the number of partial copies [split][M][round_up(N, 32)] left in splitk_ws, for a
// following kernel of the caller to sum (in split order) together with its own work; 0 = the epilogue has run.
hipError_t launch_gemm(const bf16_t* A, int lda, int M, const PackedWeight& W, const EpiArgs& epi, float* splitk_ws,
                       size_t splitk_elems, int n_cus, hipStream_t s, int* deferred_splits = nullptr);

struct AttnArgs {
  const bf16_t* q;   // [T, q_stride] rotated queries
  int q_stride;
  const bf16_t* kv;  // layer pool
  bf16_t* out;       // [T, Hq * D]
  int Hq, Hkv, D;
  float scale_log2;  // log2(e) / sqrt(D)
  const ReqInfo* reqs;
  const int32_t* visit_phys;
  const int32_t* visit_logical;
  const int32_t* visit_pairs;  // 16-byte entries (physical a, logical a, physical b, logical b); an odd tail repeats its page
  const uint32_t* mask_words;
};
hipError_t launch_attn_decode(const AttnArgs& a, const DecodeWave* waves, const int2* wave_pg, int slots,
                              const DecodeSeg* segs, const DecodeCol* cols, int n_waves, int rows_cap, float* part_o,
                              float* part_ml, bool read_once, hipStream_t s);
hipError_t launch_attn_merge(const AttnArgs& a, const int32_t* dec_reqs, int n_dec_reqs, const int32_t* mref_indptr,
                             const int32_t* mrefs, int rows_cap, const float* part_o, const float* part_ml,
                             hipStream_t s);
// pair_weights: the items' softmax weights enter the PV product as bf16 pairs hi + lo (rows that may see few keys)
hipError_t launch_attn_prefill(const AttnArgs& a, const PrefillItem* items, int n_items, bool pair_weights,
                               hipStream_t s);

// rows / tile_ad: the batch's adapter tiles (32 rows each); z: [ksplits][n_tiles * 32, 3, rmax_p] fp32, where
// ksplits (from lora_ksplits, the same for the down and the up launch of a projection group) splits the input
// dimension over workgroups when the batch has few tiles; z_rows = rows of 3 * rmax_p floats the buffer holds
int lora_ksplits(int n_tiles, int n_slots, int in, int rmax_p, size_t z_rows);
hipError_t launch_lora_down(const bf16_t* x, int ldx, int in, int n_tiles, int n_slots, const int32_t* rows,
                            const int32_t* tile_ad, const LoraPair* table, int layer, int n_layers, int proj0, float* z,
                            int rmax_p, int ksplits, hipStream_t s);
hipError_t launch_lora_up(void* dst, int ld, int out, int kind, int col0, int kd, int n_tiles, const int32_t* rows,
                          const int32_t* tile_ad, const LoraPair* table, int layer, int n_layers, int proj, int slot,
                          const float* z, int rmax_p, int ksplits, hipStream_t s);
hipError_t launch_swiglu_f32(const float* gu, int I, bf16_t* act, int T, hipStream_t s);

int topk_chunks(int V, int k);  // chunks per row used by launch_topk (<= 16), 0 if unsupported
// cand_ws: [n, chunks, k] 64-bit candidates; stats_ws: [n, chunks, 2] floats
hipError_t launch_topk(const float* logits, int n, int V, int k, float inv_temp, int32_t* out_ids, float* out_probs,
                       unsigned long long* cand_ws, float* stats_ws, hipStream_t s);
