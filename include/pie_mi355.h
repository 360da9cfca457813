/*
 * pie_mi355 - C ABI of the inference-layer hot path of a programmable LLM serving system on one
 * AMD MI355X (gfx950): the batched `forward` handler (one Llama-class decoder layer applied to a
 * heterogeneous batch of commands against KvPage page tables with per-token attention masks and
 * KV append) and the `get_next_dist` handler (next-token distribution truncated to top-K).
 *
 * Conventions for every call
 *   - "host" pointers are ordinary CPU memory owned by the caller and read only during the call.
 *   - "dev" pointers are device memory on the GPU the context was created on, owned by the
 *     caller; the library reads/writes them on the context's stream.
 *   - bf16 tensors are raw 16-bit patterns.  Nothing here is a torch type.
 *   - All GPU work is enqueued on the HIP stream given to pie_create and is complete only after
 *     pie_synchronize (or a stream synchronisation by the caller).
 *   - Every call returns a pie_status; on error nothing has been launched for that call unless
 *     stated otherwise, and pie_last_error gives a message.  The library never aborts.
 *   - One context <-> one stream <-> one GPU.  A context is not thread-safe.
 */
#ifndef PIE_MI355_H
#define PIE_MI355_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pie_ctx pie_ctx;     /* owns the Embed pool, the KvPage pool, packed weights, workspace */
typedef struct pie_batch pie_batch; /* a validated forward batch resident on the device */
typedef int32_t pie_status;

enum {
  PIE_OK = 0,
  PIE_EINVAL = -1,       /* null pointer, bad shape, non-positive temperature, ... */
  PIE_ERANGE = -2,       /* page id, embed id, slot, layer or top_k out of range */
  PIE_EBATCH = -3,       /* more tokens or requests than the context was sized for */
  PIE_ECONFLICT = -4,    /* two tokens of one batch write the same (page, slot) */
  PIE_ENOMEM = -5,       /* device allocation failed */
  PIE_EHIP = -6,         /* a HIP call failed (asynchronous faults surface at pie_synchronize) */
  PIE_EUNSUPPORTED = -7  /* shape outside what the kernels are built for */
};

/* Model shape: a Llama-family decoder layer (Implementation section: the handlers support the
 * Llama family) - RMSNorm, grouped-query attention with rotary positions, SwiGLU MLP, no biases.
 * Supported: head_dim 64 or 128, page_size 16 or 32 (KvPage sizes of 8-32 tokens are named in the
 * Resources paragraph; a page of 32 is stored as two consecutive 16-token blocks, and the page counts
 * and page bytes reported by pie_batch_work are then in 16-token blocks), n_q_heads a multiple of
 * n_kv_heads with ratio <= 8, hidden / mlp_dim / vocab multiples of 32. */
typedef struct {
  int32_t hidden, n_q_heads, n_kv_heads, head_dim, mlp_dim, vocab, page_size;
  float rms_eps, rope_theta;
  int32_t n_layers; /* layers resident in this context (weights + one KvPage pool each) */
} pie_model_desc;

/* Resource pools, sized once at start-up (Control layer, Resource management: a global pool of
 * Embed and KvPage resources physically located in the inference layer). */
typedef struct {
  int32_t n_kv_pages, n_embeds, max_batch_tokens, max_batch_requests, max_top_k, max_dist_rows;
  int32_t max_adapters, max_lora_rank; /* LoRA adapters (pie_load_adapter); both 0 = none */
} pie_pool_desc;

/* Create a context on the current HIP device (System Architecture, Inference layer: the handlers own the resource
 * pools and a workspace set up once at start; API handlers: a native handler with pre-allocated buffers).
 * `hip_stream` is a hipStream_t (NULL = default stream).  Allocates pools (zero-filled) and workspace; nothing is allocated afterwards by
 * pie_forward / pie_get_next_dist. */
pie_status pie_create(const pie_model_desc* model, const pie_pool_desc* pool, void* hip_stream, pie_ctx** out);
pie_status pie_destroy(pie_ctx* ctx);
/* A context that only deserialises and plans batches (Batch scheduler: the batch is validated and turned into the
 * handler's work lists before anything is launched): no HIP call is made, nothing is allocated on a device, so it
 * also works on a machine without a GPU.  `wave_slots` stands for the number of waves the decode-attention kernel
 * keeps resident (8 per compute unit: 2048 on MI355X).  pie_batch_create (all its checks and error codes),
 * pie_batch_work, pie_batch_destroy, pie_mask_kvpage, pie_last_error and pie_destroy work on it; every call that
 * needs the device returns PIE_EINVAL.  For schedulers that want the cost of a batch before committing to it, and
 * for tests of the host logic. */
pie_status pie_create_planner(const pie_model_desc* model, const pie_pool_desc* pool, int32_t wave_slots,
                              pie_ctx** out);
/* Message of the last failing call on ctx (ctx may be NULL for pie_create failures); storage
 * is owned by the library and valid until the next call. */
const char* pie_last_error(const pie_ctx* ctx);

/* Weights: dev pointers, bf16, Linear layout [out, in]; gains [hidden].  The library copies them
 * into its own tiled storage, so the caller may free its tensors once the stream has drained. */
pie_status pie_load_layer(pie_ctx* ctx, int32_t layer, const void* g1, const void* wq, const void* wk,
                          const void* wv, const void* wo, const void* g2, const void* wgate, const void* wup,
                          const void* wdown);
/* g_final may be NULL: get_next_dist then applies no final norm. */
pie_status pie_load_head(pie_ctx* ctx, const void* g_final, const void* w_lm /* [vocab, hidden] */);

/* `forward_with_adapter` (Forward API: a call may name LoRA adapters to serve fine-tuned models).  An adapter is,
 * per layer and per projection, an optional pair A [rank, in], B [out, rank] (dev bf16, row-major, copied by the
 * call) and a scale: requests of a batch that name the adapter (pie_forward_batch.adapter_ids) compute
 * W x + scale * B (A x) for that projection.  rank = 0 or A = B = NULL removes the pair.  Projections: the seven
 * linear maps of the layer.  Errors: PIE_EINVAL (null with rank > 0, context created without adapters),
 * PIE_ERANGE (adapter, layer, projection or rank out of range), PIE_ENOMEM, PIE_EHIP.  Synchronises the stream. */
enum { PIE_PROJ_Q = 0, PIE_PROJ_K = 1, PIE_PROJ_V = 2, PIE_PROJ_O = 3, PIE_PROJ_GATE = 4, PIE_PROJ_UP = 5,
       PIE_PROJ_DOWN = 6, PIE_N_PROJ = 7 };
pie_status pie_load_adapter(pie_ctx* ctx, int32_t adapter, int32_t layer, int32_t projection, int32_t rank,
                            float scale, const void* A, const void* B);

/* Embedding table for `embed_txt`: dev bf16 [vocab, hidden], copied into library storage (the caller may
 * free its tensor afterwards).  Errors: PIE_EINVAL (null, context without vocab), PIE_ENOMEM, PIE_EHIP. */
pie_status pie_load_embedding(pie_ctx* ctx, const void* table);

/* `embed_txt(q, tok, pos, embs)` (Table 1, InputText; Embed API): Embed embed_ids[i] receives row
 * token_ids[i] of the embedding table, unchanged, and the sequence position positions[i], which a later
 * forward batch with positions == NULL uses for the rotary step (Forward API: the call works on the sequence
 * positions associated with its resources).  All three arrays are host int32 [n].  Synchronises the stream.
 * Errors: PIE_EINVAL (null, no table loaded), PIE_ERANGE (token id, embed id, negative position),
 * PIE_ECONFLICT (one embed id named twice). */
pie_status pie_embed_txt(pie_ctx* ctx, const int32_t* token_ids, const int32_t* positions, int32_t n,
                         const int32_t* embed_ids);

/* Resource seeding / inspection.  Stand-ins for what `embed_txt` and earlier `forward` calls
 * leave in the pools (Table 1; Embed API), used by tests and the benchmark.  ids/slots: host
 * int32 [n]; data: dev bf16.  KV rows are token-major [n, n_kv_heads, head_dim]; K is stored as
 * given (already rotated).  The pool layout itself is private to the library.  pie_embed_write leaves the
 * written Embeds without a recorded position. */
pie_status pie_embed_write(pie_ctx* ctx, const int32_t* embed_ids, int32_t n, const void* src /* dev [n, hidden] */);
pie_status pie_embed_read(pie_ctx* ctx, const int32_t* embed_ids, int32_t n, void* dst /* dev [n, hidden] */);
pie_status pie_kv_write(pie_ctx* ctx, int32_t layer, const int32_t* page_ids, const int32_t* slots, int32_t n,
                        const void* k /* dev */, const void* v /* dev */);
pie_status pie_kv_read(pie_ctx* ctx, int32_t layer, const int32_t* page_ids, const int32_t* slots, int32_t n,
                       void* k /* dev */, void* v /* dev */);

/* `mask_kvpage(q, tgt, mask)` (Table 1, Forward row: masks the KV cache in a token-level manner): sets the
 * token-level mask of each target KvPage; bit s of visible_bits[k] says whether the token in slot s of page
 * page_ids[k] stays visible (bits at and above page_size are ignored; a page of 32 tokens uses all 32 bits).  The mask replaces the page's previous
 * one, holds in every layer, and is honoured, on top of a call's own mask, by every batch deserialised
 * afterwards (pie_batch_create reads the masks; a batch created earlier keeps what it saw).  A fresh context has
 * every token visible.  Host arrays [n]; no GPU work.  Errors: PIE_EINVAL, PIE_ERANGE. */
pie_status pie_mask_kvpage(pie_ctx* ctx, const int32_t* page_ids, const uint32_t* visible_bits, int32_t n);

/* `copy_kvpage(q, src, dst)` (Table 1, Allocate row: copies KV cache contents at token level): token k is
 * read from (src_pages[k], src_slots[k]) and written to (dst_pages[k], dst_slots[k]), K and V, bit for bit,
 * in every layer.  Page masks are not copied.  Host int32 arrays [n].  No token may be written twice or be
 * both read and written by one call (PIE_ECONFLICT).  Synchronises the stream.
 * Errors: PIE_EINVAL, PIE_ERANGE, PIE_ECONFLICT, PIE_EHIP. */
pie_status pie_copy_kvpage(pie_ctx* ctx, const int32_t* src_pages, const int32_t* src_slots,
                           const int32_t* dst_pages, const int32_t* dst_slots, int32_t n);

/* One batch of `forward(q, ikv, iemb, okv, oemb, mask)` commands as the batch scheduler hands it
 * to the handler (Table 1 `forward`; Forward API; Batch scheduler: horizontal + vertical
 * batching).  The command queue argument is gone: batching has been done.  All arrays are host.
 *
 *   request r owns tokens tok_indptr[r] .. tok_indptr[r+1)  (its input Embeds, in order)
 *   page table of r: page_ids[page_indptr[r] .. page_indptr[r+1)) = input KvPages followed by
 *     output KvPages, in logical order; logical KV index j lives in page j / page_size, slot
 *     j % page_size of that list
 *   kv_len[r]: KV length AFTER this call's append; new token i of r is stored at logical index
 *     kv_len[r] - n_new_r + i, whatever its position
 *   positions[t]: explicit rotary position of token t (Forward API: explicit sequence positions); NULL
 *     takes, for every token, the position recorded with its input Embed by pie_embed_txt (PIE_EINVAL
 *     when an input Embed carries none)
 *   out_embed_ids[t]: Embed that receives the layer output of token t, or -1 to drop the row
 *     (fewer output than input Embeds: the example with 9 inputs and 1 output).  An Embed may be
 *     both input and output of one call (autoregressive-loop example).
 *   mask: boolean matrix, one row per new token over logical KV index [0, kv_len[r]) including
 *     the tokens appended by this call; row = ceil(kv_len[r]/32) uint32 words, bit (j % 32) of
 *     word j / 32, LSB first, bits >= kv_len ignored.  mask_indptr (word offsets, [R+1]) may be
 *     NULL, and a request with an empty word range has its mask inferred: causal on logical
 *     order (token i sees j <= kv_len - n_new + i).  A row with no visible key outputs zeros.
 *
 *   adapter_ids[r]: the LoRA adapter request r runs with (`forward_with_adapter`), see pie_load_adapter
 *
 * Effects of a call, in order: read all input Embeds; append every new K/V; attend; write output
 * Embeds.  Two tokens of one batch must not write the same (page, slot) (vertical batching is
 * only done when calls do not conflict); checked when validate != 0.
 */
typedef struct {
  int32_t n_requests, n_tokens;
  const int32_t* tok_indptr;    /* [R+1] */
  const int32_t* in_embed_ids;  /* [T] */
  const int32_t* out_embed_ids; /* [T] */
  const int32_t* positions;     /* [T] or NULL */
  const int32_t* page_indptr;   /* [R+1] */
  const int32_t* page_ids;      /* [page_indptr[R]] */
  const int32_t* kv_len;        /* [R] */
  const int64_t* mask_indptr;   /* [R+1] or NULL */
  const uint32_t* mask_words;   /* [mask_indptr[R]] or NULL */
  const int32_t* adapter_ids;   /* [R] LoRA adapter of each request, -1 = none; NULL = no request has one */
} pie_forward_batch;

/* Deserialise a batch: check shapes and id ranges on the host (validate != 0 adds the
 * write-conflict check), derive the attention work lists (pages with no visible key are
 * dropped, so cost follows the mask and not the context length), and copy everything the
 * kernels need to the device.  Allocates device memory owned by the returned pie_batch.
 * Errors: PIE_EINVAL, PIE_ERANGE, PIE_EBATCH, PIE_ECONFLICT, PIE_ENOMEM, PIE_EHIP. */
pie_status pie_batch_create(pie_ctx* ctx, const pie_forward_batch* batch, int32_t validate, pie_batch** out);
pie_status pie_batch_destroy(pie_ctx* ctx, pie_batch* batch);

/* A batch runs only on the context that created it: the forward calls and pie_batch_destroy return PIE_EINVAL for a
 * batch of another context, and the forward calls for a batch made by a planning context (it has no device block). */

/* Run one decoder layer over the batch (Forward API: attention and transformation steps):
 * RMSNorm, QKV projection, rotary step + KV append into pages, paged masked GQA attention,
 * output projection + residual, RMSNorm, SwiGLU MLP + residual, output Embeds.  Enqueues only;
 * allocates nothing.  The batch may be reused across calls and layers. */
pie_status pie_forward(pie_ctx* ctx, int32_t layer, const pie_batch* batch);

/* The same call through every layer of the model (Forward API: the core Transformer forward pass; the
 * autoregressive-loop example): layer l appends to and attends over its own KvPage pool with the batch's
 * page table, its input is the output of layer l-1 (kept in fp32 between layers), layer 0 reads the input
 * Embeds and the last layer stores the output Embeds as bf16.  Every layer must be loaded.  Enqueues only;
 * allocates nothing.  Errors: PIE_EINVAL (null, a layer without weights), PIE_EBATCH, PIE_EHIP. */
pie_status pie_forward_all(pie_ctx* ctx, const pie_batch* batch);

/* Convenience: pie_batch_create + pie_forward + pie_batch_destroy (synchronises the stream). */
pie_status pie_forward_host(pie_ctx* ctx, int32_t layer, const pie_forward_batch* batch, int32_t validate);

/* forward and sampling in one call (the paper measures the cost of sampling that is not pipelined behind the
 * forward pass: Evaluation, overhead breakdown): pie_forward_all over the batch, then get_next_dist on the
 * output Embeds of the batch's token rows rows[0..n) (host int32; each must name an output Embed), all enqueued
 * back to back on the context's stream without any host synchronisation.  Arguments as for pie_get_next_dist;
 * all of them are checked before anything is enqueued.  (The two separate calls are stream-ordered in the same
 * way; this entry point only saves the caller the id bookkeeping.) */
pie_status pie_forward_dist(pie_ctx* ctx, const pie_batch* batch, const int32_t* rows, int32_t n, int32_t top_k,
                            float temperature, int32_t* out_ids, float* out_probs);

/* `get_next_dist(q, emb) -> Dist` for n Embeds (Table 1; Sample API): final RMSNorm when the head
 * has a gain, LM head in fp32 logits, softmax(logits / temperature) over the whole vocabulary,
 * truncated to the top_k entries (Sample API: top-K truncation, K configurable, default 256).
 * Output per row: ids and probabilities by descending probability, equal values by ascending id;
 * probabilities are those of the full distribution (no renormalisation).
 * embed_ids: host int32 [n]; out_ids dev int32 [n, top_k]; out_probs dev float [n, top_k].
 * Errors: PIE_EINVAL (temperature <= 0, n <= 0), PIE_ERANGE (top_k, ids), PIE_EBATCH (n). */
pie_status pie_get_next_dist(pie_ctx* ctx, const int32_t* embed_ids, int32_t n, int32_t top_k, float temperature,
                             int32_t* out_ids, float* out_probs);

/* pie_get_next_dist for callers that cannot allocate device memory or have it allocated on their behalf: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the
 * same result as pie_get_next_dist, for at most 32 rows and top_k <= 1024; every intermediate (the staged ids,
 * normalised rows, fp32 logits, split-K partial sums, top-k candidates and chunk statistics) lives in one
 * file-scope device array of 16 MiB that each GPU the library runs on holds until the process ends, and the embed
 * ids reach the device as kernel arguments, so the call makes no hipMalloc, hipFree, copy from pageable memory or
 * other allocating library call.  n x vocab x 4 bytes of logits, n x 16 x top_k x 8 bytes of candidates and
 * n x hidden x 2 bytes of normalised rows must fit the array (at a vocabulary of 128256 and top_k 256: up to 30
 * rows); otherwise PIE_EBATCH, as for n > 32.
 * Every call on a GPU, from any context, uses that GPU's one array and leaves its contents behind (no kernel relies
 * on them): calls that overlap on one GPU (two contexts on two streams) race and must be serialised by the caller.
 * Other errors as pie_get_next_dist. */
pie_status pie_get_next_dist_static(pie_ctx* ctx, const int32_t* embed_ids, int32_t n, int32_t top_k,
                                    float temperature, int32_t* out_ids, float* out_probs);

/* Waits for the context's stream (Table 1, `synchronize`: completion of the calls issued so far). */
pie_status pie_synchronize(pie_ctx* ctx);

/* ---- observation points for parity tests and per-kernel timing (not part of the serving path).  These are test
 *      and measurement hooks of this library; no passage of the paper describes them. ---- */

/* Copy an intermediate of the last pie_forward / pie_get_next_dist to `dst` (dev).  Sizes in
 * elements: Q [T, Hq*D] bf16 (after the rotary step), ATTN [T, Hq*D] bf16, RESID [T, hidden]
 * fp32 (after the attention block), ACT [T, mlp_dim] bf16, LOGITS [n, vocab] fp32. */
enum { PIE_TAP_Q = 0, PIE_TAP_ATTN = 1, PIE_TAP_RESID = 2, PIE_TAP_ACT = 3, PIE_TAP_LOGITS = 4 };
pie_status pie_read_tap(pie_ctx* ctx, int32_t which, void* dst, int64_t n_elements);

/* Stage timing.  When enabled, pie_forward / pie_get_next_dist bracket each stage with HIP events
 * on the context's stream; pie_stage_times synchronises and returns the milliseconds of the last
 * call per stage (host float[PIE_N_STAGES]; 0 for stages that did not run). */
enum {
  PIE_STAGE_NORM1 = 0, PIE_STAGE_QKV = 1, PIE_STAGE_ROPE_APPEND = 2, PIE_STAGE_ATTN_DECODE = 3,
  PIE_STAGE_ATTN_PREFILL = 4, PIE_STAGE_ATTN_MERGE = 5, PIE_STAGE_OPROJ = 6, PIE_STAGE_NORM2 = 7,
  PIE_STAGE_GATEUP = 8, PIE_STAGE_DOWN = 9, PIE_STAGE_HEAD_NORM = 10, PIE_STAGE_LM_HEAD = 11,
  PIE_STAGE_TOPK = 12, PIE_N_STAGES = 13
};
pie_status pie_set_stage_timing(pie_ctx* ctx, int32_t enabled);
pie_status pie_stage_times(pie_ctx* ctx, float* ms_out);

/* Algorithmic work of a batch for roofline accounting: out[0] = KV bytes the attention stage has
 * to read (visible pages x page bytes, K and V, all kv heads, counted per request), out[1] = decode-path
 * share of out[0], out[2] = attention flops (QK^T and PV over visible pages), out[3] = number of visited
 * (request, page) pairs, out[4] = page bytes of the distinct physical pages visited by the decode-path requests
 * (what HBM has to deliver to them when pages are shared), out[5] = KV bytes the decode kernel asks for after requests
 * that share pages have been grouped (<= out[1]).  Host int64[6]. */
pie_status pie_batch_work(const pie_batch* batch, int64_t* out);

/* Shape of the launch plan of a batch: out[0] = waves of the decode-attention kernel, out[1] = segments (runs of
 * one (column group, kv head) inside a wave's share; one partial row set each), out[2] = page pairs a wave's share
 * holds at most, out[3] = workgroup rows of the prefill kernel ((request, 32-token query block) items), out[4] =
 * requests on the decode path, out[5] = query columns per segment the partial buffers are sized for (at most 16;
 * more than one request's rows when requests that share pages are walked together), out[6] and out[7] = workgroups
 * of the first and the second prefill launch (see pie_batch_prefill_work).
 * Host int64[8]. */
pie_status pie_batch_plan_info(const pie_batch* batch, int64_t* out);

/* The prefill attention launches of a batch, as the planner laid them out: one entry per workgroup in launch order,
 * three values each (request, 32-token query block, kv head); request -1 marks an empty slot.  There are two
 * launches, listed one after the other (their sizes: pie_batch_plan_info out[6], out[7], both multiples of 8): the
 * second holds the query blocks whose rows may see only a few keys (requests with a bitmap; blocks of causal
 * requests that start within the first 64 keys) and runs with the softmax weights held as bf16 pairs.  Workgroup i
 * of a launch runs on XCD i % 8 (the hardware's round-robin), and within a launch the planner puts all query blocks
 * of one (request, kv head) on one XCD (System Architecture, Inference layer: how a batch of API calls is executed is the handler's business;
 * this is its layout on this chip, exposed for the
 * host-logic tests).  Copies at most cap entries into out (host int32[cap * 3]) and stores the total number of
 * entries in *n_entries.  Works on planner contexts. */
pie_status pie_batch_prefill_work(const pie_batch* batch, int32_t* out, int32_t cap, int32_t* n_entries);

#ifdef __cplusplus
}
#endif
#endif /* PIE_MI355_H */
