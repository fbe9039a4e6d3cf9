/*
 * hcache.h -- C ABI of the MI355X-native HCache restoration library (libhcache.so).
 *
 * What the library does (paper Section 3.1): a serving system saves, per transformer
 * layer, the hidden state that enters the layer for every token of a context.  To
 * restore that context's KV cache it fetches the saved states of layer L from host
 * storage and re-projects them: K = W_k * H, V = W_v * H.  The equations of the
 * paper leave out the layer's input normalisation and the position embedding
 * (Section 2.1); Section 5 names the device steps: a GEMM, then a kernel that
 * applies RoPE to the re-projected keys and copies K/V into the (paged, Section 6
 * "Baselines") KV cache.  Fetching layer L+1 overlaps the projection of layer L
 * (Section 3.1, pipelined restoration; Section 5, "Pipelined state transmission").
 * Host-side, the saved states live in fixed-size token chunks per layer (Section
 * 4.2.1).
 *
 * Here every device step of one layer -- RMSNorm with the layer's gain, the fused
 * K|V projection on bf16 matrix cores with fp32 accumulation, RoPE on K at each
 * token's absolute position, one round-to-nearest-even conversion to bf16 and the
 * scatter into block-table pages -- is ONE kernel launch.
 *
 * Conventions
 *   - No exception crosses this boundary.  Every call returns an hc_status; on failure
 *     hc_last_error() holds a message for the calling thread.
 *   - "d_" arguments are DEVICE pointers (HBM) owned by the caller; "h_" arguments are
 *     HOST pointers.  Device pointers must be 16-byte aligned (HC_EALIGN otherwise).
 *   - `stream` arguments are hipStream_t values passed as void* (NULL = the null stream).
 *     Launches are asynchronous on that stream; the library never synchronises a
 *     caller's stream except where a function says so.
 *   - All matrices are row-major; bf16 is the upper half of an IEEE binary32.
 *   - A context (hc_ctx) belongs to the device that was current in hc_create and may be
 *     used by one host thread at a time.
 *   - Rows whose position cannot be mapped (outside the block table, unmapped block,
 *     page outside the pool, position >= max_position) are SKIPPED, never written out of
 *     bounds, and raise a sticky flag readable with hc_poll_device_error.
 */
#ifndef HCACHE_H
#define HCACHE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t hc_status;
enum {
  HC_OK      = 0,
  HC_EINVAL  = -1,  /* bad argument (null pointer, shape the kernels do not support)   */
  HC_ERANGE  = -2,  /* index outside its table (layer, chunk, token range, capacity)   */
  HC_EALIGN  = -3,  /* device pointer not 16-byte aligned                              */
  HC_ENOMEM  = -4,  /* host or device allocation failed                                */
  HC_EHIP    = -5,  /* a HIP runtime call failed; message carries hipGetErrorString    */
  HC_ESTATE  = -6   /* call out of order (weights/pool not set, layer order in store)  */
};

/* bits of the sticky device error word */
enum {
  HC_DEV_BAD_POSITION = 1,  /* position < 0, >= max_position, or beyond the block table */
  HC_DEV_BAD_PAGE     = 2   /* block table entry < 0 or >= num_pages                   */
};

typedef struct hc_ctx hc_ctx;
typedef struct hc_store hc_store;
typedef struct hc_saver hc_saver;

/* Shape of the model whose KV cache is restored.  Supported by the kernels:
 * d_model % 64 == 0, head_dim % 64 == 0, block_size a power of two, n_q_heads % n_kv_heads
 * == 0.  rope_style 0 pairs feature i with i + head_dim/2, 1 pairs 2i with 2i+1 (the
 * paper only cites RoFormer; both conventions are in use), 2 applies no rotation (models
 * with learned absolute position embeddings such as OPT, one of the paper's test models,
 * Section 6 "Models"; positions then only address the cache).  The RoPE table is built for
 * positions [0, max_position).  norm_kind selects the layer's input normalisation:
 * HC_NORM_RMS (x / sqrt(mean x^2 + eps) * gain) or HC_NORM_LAYER ((x - mean) / sqrt(var + eps)
 * * gain + shift, biased variance); rms_eps is the eps of either. */
enum { HC_NORM_RMS = 0, HC_NORM_LAYER = 1 };
typedef struct {
  int32_t n_layers;
  int32_t d_model;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;
  int32_t block_size;
  int32_t max_position;
  int32_t rope_style;
  float   rope_theta;
  float   rms_eps;
  int32_t norm_kind;
} hc_model_desc;

/* Message describing the last failure on the calling thread ("" if none). */
const char* hc_last_error(void);

/* Library version string, e.g. "hcache-mi355x 0.1". */
const char* hc_version(void);

/* Validate `desc` only (no device work): HC_OK or HC_EINVAL with a message. */
hc_status hc_validate_desc(const hc_model_desc* desc);

/* Create a context on the current device.  Allocates the fp32 (cos, sin) RoPE table
 * [max_position][head_dim/2] and fills it with an fp64-evaluated kernel; synchronises
 * the null stream once.  *out is NULL on failure. */
hc_status hc_create(const hc_model_desc* desc, hc_ctx** out);

/* Free everything the context owns (packed weights, RoPE table, staging buffers).
 * Synchronises the device first. */
hc_status hc_destroy(hc_ctx* ctx);

/* Give the context one layer's projection weights.
 *   d_wkv   bf16 [2*d_kv, d_model]  nn.Linear layout; rows [0,d_kv) = W_k, [d_kv,2 d_kv) = W_v
 *   d_gamma bf16 [d_model]          gain of the layer's input RMSNorm
 * The library allocates its own device copy in the matrix-core friendly order it needs
 * (gamma folded into the weights, one bf16 rounding) with a kernel on `stream`; the
 * caller's buffers may be reused once `stream` has passed that point.  Calling it again
 * for the same layer replaces the weights. */
hc_status hc_set_layer_weights(hc_ctx* ctx, int32_t layer, const void* d_wkv,
                               const void* d_gamma, void* stream);

/* The same for layers with additive terms (OPT-style: LayerNorm shift and projection biases;
 * RMSNorm models with K/V biases):
 *   d_beta bf16 [d_model]  shift of the input LayerNorm; NULL = none; must be NULL under
 *                          HC_NORM_RMS (HC_EINVAL)
 *   d_bias bf16 [2*d_kv]   bias of the K then the V projection; NULL = none
 * K = W_k * norm(x) + b_k (then rotated unless rope_style = 2), V = W_v * norm(x) + b_v.  The
 * library folds the additive terms into one fp32 constant per output feature. */
hc_status hc_set_layer_weights_affine(hc_ctx* ctx, int32_t layer, const void* d_wkv,
                                      const void* d_gamma, const void* d_beta,
                                      const void* d_bias, void* stream);

/* Register one layer's paged KV pool (borrowed, never freed by the library):
 *   d_pool bf16 [num_pages][2 (0=K,1=V)][block_size][n_kv_heads][head_dim]
 * num_pages * 2 * block_size must stay below 2^31 (HC_ERANGE). */
hc_status hc_set_kv_pool(hc_ctx* ctx, int32_t layer, void* d_pool, int64_t num_pages);

/* Restore layer `layer` of ONE context from hidden states already in HBM
 * (Section 3.1 equations + Section 5 RoPE/copy step).
 *   d_hidden      bf16  [n_tok, d_model]  saved inputs of the layer (before its RMSNorm)
 *   d_positions   int32 [n_tok]           absolute positions; drive RoPE and the slot:
 *                                         page = block_table[pos / block_size],
 *                                         slot = pos % block_size
 *   d_block_table int32 [n_blocks]        logical block -> page of the layer's pool
 * n_tok == 0 is a no-op.  One asynchronous launch on `stream`. */
hc_status hc_restore_kv(hc_ctx* ctx, int32_t layer, const void* d_hidden,
                        const int32_t* d_positions, int32_t n_tok,
                        const int32_t* d_block_table, int32_t n_blocks, void* stream);

/* The same for layers [layer_begin, layer_begin + n_layers) of one context whose saved inputs
 * are ALL resident in HBM: h_d_hidden is a HOST array of n_layers device pointers, entry i =
 * bf16 [n_tok, d_model] of layer layer_begin + i; positions and block table are shared (one
 * context).  The layers go out in launches of up to 8 layers each (for short contexts, whose
 * layers have fewer than 32 tiles of 256 features x 256 tokens: as many layers as fill the 256
 * compute units once, up to 32), which removes the gaps between per-layer kernels and lets the
 * compute units run out of step.
 * Per layer the result is identical to hc_restore_kv's.  Every layer needs weights and a
 * pool (HC_ESTATE).  The pointer array is read during the call only. */
hc_status hc_restore_kv_layers(hc_ctx* ctx, int32_t layer_begin, int32_t n_layers,
                               const void* const* h_d_hidden, const int32_t* d_positions,
                               int32_t n_tok, const int32_t* d_block_table, int32_t n_blocks,
                               void* stream);

/* Ragged batch: the tokens of n_seq contexts concatenated into one projection.
 *   d_cu_seqlens   int32 [n_seq + 1]          context s owns rows cu[s] .. cu[s+1]-1
 *   d_block_tables int32 [n_seq][max_blocks]  one row per context, padded with -1
 * h_total_tokens must equal cu[n_seq] (the host does not read device memory). */
hc_status hc_restore_kv_ragged(hc_ctx* ctx, int32_t layer, const void* d_hidden,
                               const int32_t* d_positions, int32_t h_total_tokens,
                               const int32_t* d_cu_seqlens, int32_t n_seq,
                               const int32_t* d_block_tables, int32_t max_blocks,
                               void* stream);

/* Read and clear the sticky device error word (HC_DEV_* bits).  Synchronises `stream`
 * so that every launch queued on it has reported. */
hc_status hc_poll_device_error(hc_ctx* ctx, void* stream, int32_t* out_flags);

/* ---- host store of saved hidden states (Section 4.2.1, read side) -------------------
 * A pinned host arena cut into chunks of `chunk_tokens` rows of d_model bf16; the
 * states of (context, layer) are a list of chunks, the last one possibly part filled.
 * Chunks are taken from the arena in the order the data arrives, i.e. in generation
 * order (layer-before-token, Section 3.2 "C2"); restoration reads them one layer at a
 * time through the index.  The index is guarded by a lock, so appends (also through a saver),
 * drops, queries and restores of DIFFERENT contexts may run on different host threads; one
 * context must not be appended to, dropped or restored concurrently, and its chunks must stay
 * in the store until the copies a restore has queued are complete. */
hc_status hc_store_create(int32_t n_layers, int32_t d_model, int32_t chunk_tokens,
                          int64_t capacity_chunks, hc_store** out);
/* Same, choosing the arena's memory: pinned != 0 -> hipHostMalloc (what asynchronous,
 * full-rate host->HBM copies need; HC_ENOMEM if the runtime cannot provide it);
 * pinned == 0 -> ordinary page-aligned host memory (hosts without a GPU; copies from it
 * go through the runtime's pageable path).  hc_store_create is pinned = 1. */
hc_status hc_store_create_ex(int32_t n_layers, int32_t d_model, int32_t chunk_tokens,
                             int64_t capacity_chunks, int32_t pinned, hc_store** out);
hc_status hc_store_destroy(hc_store* store);

/* Append n_tok rows (h_rows: host bf16 [n_tok, d_model]) to (seq_id, layer).  Layers
 * must not run ahead of the layer below them (HC_ESTATE).  HC_ERANGE when the arena is
 * full.  Plain host memcpy. */
hc_status hc_store_append(hc_store* store, int64_t seq_id, int32_t layer,
                          const void* h_rows, int32_t n_tok);

/* Tokens stored for (seq_id, layer); 0 for an unknown context. */
int64_t hc_store_tokens(const hc_store* store, int64_t seq_id, int32_t layer);

/* Read-side index: pointer to chunk `chunk` of (seq_id, layer) in pinned host memory and
 * the number of valid rows in it. */
hc_status hc_store_chunk(const hc_store* store, int64_t seq_id, int32_t layer,
                         int32_t chunk, const void** h_ptr, int32_t* rows);

/* Forget a context and return its chunks to the arena. */
hc_status hc_store_drop(hc_store* store, int64_t seq_id);

/* Restore ALL layers of tokens [tok_begin, tok_begin + n_tok) of one stored context,
 * token i sitting at absolute position pos_offset + i (Section 3.1 pipeline; Section 5
 * "Pipelined state transmission").  Per layer the chunks are copied to one of two HBM
 * staging buffers -- by the copy engines, one (strided) hipMemcpy2DAsync per run of equally
 * spaced chunks, even layers on `copy_stream` and odd layers on a second copy stream the
 * context owns (so that the fixed cost of one transfer overlaps the bytes of the other), or by
 * a gather kernel on `copy_stream` that reads the pinned arena over the host link
 * (hc_set_loader) -- and the restoration kernel runs on `compute_stream`; events order them so
 * that the transfer of layer L+1 overlaps the kernel of layer L.  Staging buffers (and the
 * second stream) are created inside the call when the context has none.  Returns after
 * everything is enqueued; every copy is complete once `compute_stream` has run dry, which is
 * what the caller synchronises (not `copy_stream` alone) before it changes the store.  The two
 * streams must differ. */
hc_status hc_restore_context(hc_ctx* ctx, const hc_store* store, int64_t seq_id,
                             int32_t tok_begin, int32_t n_tok, int32_t pos_offset,
                             const int32_t* d_block_table, int32_t n_blocks,
                             void* compute_stream, void* copy_stream);

/* Test hook: fill both staging buffers of the context with a bf16 NaN pattern (0x7FFF), on
 * `compute_stream` after everything queued there, and make the next restore's copies wait for
 * the fill.  A restore that afterwards reads any staging row it did not copy itself produces
 * NaNs, which the parity tests detect.  HC_ESTATE before the first hc_restore_context*. */
hc_status hc_poison_staging(hc_ctx* ctx, void* compute_stream);

/* hc_restore_context for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Identical arguments, loader
 * (copy engines), kernel and result; the two staging buffers are the halves of a
 * device-resident array inside the library (2 x HC_STATIC_STAGE_BYTES, held by every GPU the
 * library runs on until the process ends), whose address and handshake events hc_create sets
 * up once per device.  The call itself calls no hipMalloc / hipFree / event creation and makes
 * no host heap allocation on the success path.  Limits: n_tok * d_model * 2 bytes <=
 * HC_STATIC_STAGE_BYTES (HC_ERANGE beyond; restore a longer range in pieces), at most 256
 * copy-engine transfers per layer (HC_ERANGE), per-launch timing off (HC_ESTATE).  The array
 * is shared by every context on a GPU and keeps the last call's rows; nothing in it has to
 * start at zero (each call overwrites the rows it reads).  Host calls are serialised by a
 * lock and a call's copies wait for the kernels of the previous call through the per-device
 * events, but two restores that are in flight on one GPU at the same time through OTHER
 * means (another process image of the library, a captured graph replayed beside a live call)
 * race on the array. */
#define HC_STATIC_STAGE_BYTES (8 * 1024 * 1024)
hc_status hc_restore_context_static(hc_ctx* ctx, const hc_store* store, int64_t seq_id,
                                    int32_t tok_begin, int32_t n_tok, int32_t pos_offset,
                                    const int32_t* d_block_table, int32_t n_blocks,
                                    void* compute_stream, void* copy_stream);
/* HC_STATIC_STAGE_BYTES as the built library has it. */
int64_t hc_static_stage_bytes(void);

/* The same for SEVERAL stored contexts at once (the restoration phase of a batch of requests,
 * Section 5 "Request scheduling"): tokens [0, h_n_tok[i]) of context h_seq_ids[i], i < n_seq,
 * at positions 0 .. h_n_tok[i] - 1.  Per layer the chunks of all contexts are copied into one
 * staging buffer, context after context, and ONE ragged launch projects them (as
 * hc_restore_kv_ragged; d_block_tables is int32 [n_seq][max_blocks], rows padded with -1).
 * The two host arrays are read during the call only.  Always uses the copy engines. */
hc_status hc_restore_contexts(hc_ctx* ctx, const hc_store* store, int32_t n_seq,
                              const int64_t* h_seq_ids, const int32_t* h_n_tok,
                              const int32_t* d_block_tables, int32_t max_blocks,
                              void* compute_stream, void* copy_stream);

/* ---- KV-offload complement (Section 4.1.2; Figure "Two ways to combine ... with KV
 * offload", layer-wise partition) ---------------------------------------------------------
 * Layers that the partition assigns to KV offload keep their KV cache on the host as token
 * rows: bf16 [n_tok][K row | V row], 2 * d_kv wide, K as it sits in the cache (rotated).
 * A KV-row store is an ordinary hc_store created with d_model = 2 * d_kv and as many layers
 * as are offloaded.
 *
 * hc_gather_kv reads the rows of the given positions out of layer `layer`'s pool into
 * d_rows (device, 16-byte aligned, n_tok * 2 * d_kv bf16): the saving direction.
 * hc_scatter_kv writes such rows into the pages the block table names: the restoring
 * direction.  Both are byte copies (bit-exact), asynchronous on `stream`; invalid rows are
 * skipped and flagged exactly as in hc_restore_kv. */
hc_status hc_gather_kv(hc_ctx* ctx, int32_t layer, void* d_rows, const int32_t* d_positions,
                       int32_t n_tok, const int32_t* d_block_table, int32_t n_blocks,
                       void* stream);
hc_status hc_scatter_kv(hc_ctx* ctx, int32_t layer, const void* d_rows,
                        const int32_t* d_positions, int32_t n_tok, const int32_t* d_block_table,
                        int32_t n_blocks, void* stream);

/* hc_restore_context with a layer-wise partition: layers [0, l_h) are restored from
 * `hidden_store` (at least l_h layers, rows d_model wide; may be NULL when l_h = 0) by the
 * restoration kernel, layers [l_h, n_layers) from `kv_store` (exactly n_layers - l_h layers,
 * rows 2 * d_kv wide, its layer j = model layer l_h + j; may be NULL when l_h = n_layers) by
 * a row-to-page copy.  Transfers run in layer order on `copy_stream`, so the hidden states
 * stream first and the offloaded KV fills the time the link would otherwise idle while the
 * projections finish.  Needs weights only for the first l_h layers.  Everything else as
 * hc_restore_context. */
hc_status hc_restore_context_mixed(hc_ctx* ctx, const hc_store* hidden_store,
                                   const hc_store* kv_store, int32_t l_h, int64_t seq_id,
                                   int32_t tok_begin, int32_t n_tok, int32_t pos_offset,
                                   const int32_t* d_block_table, int32_t n_blocks,
                                   void* compute_stream, void* copy_stream);

/* ---- two-stage saving of new hidden states (Section 4.2.2; Section 5 "Pipelined state
 * transmission", "Storage management") -------------------------------------------------
 * Stage 1: the inputs of one layer for the whole running batch (rows of several contexts
 * under continuous batching) are snapshot with ONE device->host copy into a pinned slot.
 * Stage 2: the save call itself books the rows into the chunk lists of their (context,
 * layer) -- order rule, capacity and chunk slots, in call order (layer-before-token order is
 * the caller's call order: layer 0 of a step first) -- and daemon threads copy the rows into
 * those places once the snapshot copy has completed, piece i on thread i mod n_threads.
 * While a context is being saved its chunks must not be read; hc_saver_flush makes
 * everything queued so far visible.
 *   max_rows   largest batch (rows) of one call;  n_slots  snapshots that may be in flight
 *   before hc_saver_save_layer blocks;  n_threads  daemon threads (the paper uses 8).
 * The store must outlive the saver.  One producer thread at a time. */
hc_status hc_saver_create(hc_store* store, int32_t max_rows, int32_t n_slots, int32_t n_threads,
                          hc_saver** out);
/* Waits for queued snapshots, stops the daemon threads, frees the slots. */
hc_status hc_saver_destroy(hc_saver* saver);

/* Snapshot d_hidden (device bf16 [n_rows, d_model], the inputs of `layer` for this step) and
 * queue it for the daemons; h_row_seq (host int64 [n_rows]) names the context of every row
 * and is copied by the call.  The copy runs on `down_stream` after everything queued on
 * `compute_stream` so far; `compute_stream` is made to wait for the copy, so kernels queued
 * later may overwrite the buffer (the event discipline of Section 5).  Returns once enqueued;
 * blocks only while all snapshot slots are in flight.  HC_ERANGE when the arena cannot take
 * the batch, HC_ESTATE when a layer would run ahead of the layer below it: then nothing of
 * the batch is queued (rows of contexts booked before the failing one stay counted: drop
 * those contexts). */
hc_status hc_saver_save_layer(hc_saver* saver, int32_t layer, const void* d_hidden, int32_t n_rows,
                              const int64_t* h_row_seq, void* compute_stream, void* down_stream);

/* The same without the wait on `compute_stream`: the layer whose inputs are being snapshot
 * keeps running beside the copy, and the caller calls hc_saver_fence(saver, stream) before the
 * first operator that overwrites the buffer -- in the paper's pipeline the first operator of
 * the NEXT layer (Section 5 "Pipelined state transmission").  hc_saver_fence makes `stream`
 * wait for every snapshot copy queued so far that no stream has been made to wait for; it
 * enqueues waits only and never blocks the host.  Overwriting a buffer without the fence
 * races with its copy. */
hc_status hc_saver_save_layer_deferred(hc_saver* saver, int32_t layer, const void* d_hidden,
                                       int32_t n_rows, const int64_t* h_row_seq,
                                       void* compute_stream, void* down_stream);
hc_status hc_saver_fence(hc_saver* saver, void* stream);

/* Same for rows that already sit in host memory (stage 2 only; works without a GPU). */
hc_status hc_saver_save_layer_host(hc_saver* saver, int32_t layer, const void* h_rows,
                                   int32_t n_rows, const int64_t* h_row_seq);

/* Block until every queued snapshot has reached the store.  Returns the first error a
 * daemon thread met since the last flush (a failed wait for the snapshot copy) with its
 * message, else HC_OK. */
hc_status hc_saver_flush(hc_saver* saver);

/* ---- bubble-free layer partition (Section 4.1.2) ---------------------------------------
 * Given per-layer times measured offline on a platform -- io_h: transfer of one layer's
 * hidden states, io_kv: transfer of one layer's KV cache, c_h: projection of one layer from
 * hidden states, c_token: recomputation of one layer from tokens -- split n_layers into
 * *l_h layers restored from hidden states and *l_o layers restored by the complementary
 * method so that transfer and compute finish together:
 *   c_h >  io_h (compute-bound): complement = KV offload (*complement = HC_COMPLEMENT_KV),
 *       l_h = ceil(n * io_kv / (io_kv + c_h - io_h));
 *   c_h <= io_h (transfer-bound): complement = token recomputation (HC_COMPLEMENT_RECOMPUTE),
 *       l_h = ceil(n * c_token / (c_token + io_h - c_h));
 *   l_o = n - l_h.  Pure host arithmetic (the ceiling of the double-precision quotient, as
 * printed; no tolerance); times in any common unit, all > 0.  The closed forms
 * rest on the method's premises io_kv > io_h and c_token > c_h (hidden states are the smaller
 * transfer and the cheaper compute); inputs that break them -- e.g. a grouped-query model whose
 * KV cache is narrower than its hidden states -- return HC_EINVAL, since one of the plain
 * methods alone is then at least as fast.
 * This library restores the l_h share and the KV-offload complement (hc_restore_context_mixed);
 * token recomputation is a full forward pass and belongs to the serving engine. */
enum { HC_COMPLEMENT_KV = 0, HC_COMPLEMENT_RECOMPUTE = 1 };
hc_status hc_partition_layers(int32_t n_layers, double io_h, double io_kv, double c_h,
                              double c_token, int32_t* l_h, int32_t* l_o, int32_t* complement);

/* Loader used by hc_restore_context: 0 (default) = copy engines: chunks of a layer whose
 * arena slots are equally spaced (the usual result of saving in generation order) move in
 * ONE strided copy, irregular placements in one copy per run; the compute units stay free
 * for the restoration kernel.  1 = gather kernel reading the pinned arena directly, one
 * launch per layer (pinned stores only; reaches the link rate for any placement, but its
 * waves share compute units with the restoration kernel and slow it down). */
hc_status hc_set_loader(hc_ctx* ctx, int32_t mode);

/* Split launches (paper Section 4.1.1, "Performance considerations": how well the projection
 * uses the device depends on the token count).  The restoration kernel of a single layer
 * (hc_restore_kv, hc_restore_kv_ragged, hc_restore_context*, hc_restore_contexts) runs one
 * 256-feature x 256-token tile per workgroup and compute unit, in rounds of 256, and a last
 * round with few tiles takes as long as a full one.  mode 1 (default): when a cost model says it
 * pays (a last round at most half full, d_model of about 2048 or more), the token tiles outside
 * the full rounds are computed by several workgroups each, every one over a contiguous share
 * of d_model, into an fp32 workspace the context owns (allocated by hc_create, 66 MiB), and a
 * second launch adds the shares up in a fixed order and finishes them (normalisation, RoPE,
 * scatter).  Results are deterministic and within the same tolerance, but not bit-identical to
 * an unsplit launch (fp32 summation order).  Split launches of one context are ordered after
 * each other through an event, whatever their streams.  mode 0: never split.  mode 2: split
 * whenever the shape allows it (tests and measurements).  Launches over several layers
 * (hc_restore_kv_layers) never split. */
hc_status hc_set_split(hc_ctx* ctx, int32_t mode);
/* Host-side view of that decision for a layer of d_model, d_kv and n_tok under `mode` (no
 * device work): out_plan[8] = { 1 if split else 0, feature tiles, token tiles, token tiles
 * computed whole, tiles that are split, workgroups per split tile, workgroup slots of the whole
 * tiles (first in the grid; padding slots included), workgroups of the finishing launch }. */
hc_status hc_diag_split_plan(int32_t d_model, int32_t d_kv, int32_t n_tok, int32_t mode, int32_t* out_plan);

/* ---- measurement hooks -------------------------------------------------------------
 * Average duration in milliseconds of the restoration kernel launches (one per layer, or
 * one per group of layers under hc_restore_kv_layers) queued on
 * `stream` between hc_timing_begin and hc_timing_end, measured with HIP events on that
 * stream around every launch of this context (at most 4096 launches are recorded).
 * hc_timing_end synchronises the stream.  *out_launches receives the launch count. */
hc_status hc_timing_begin(hc_ctx* ctx);
hc_status hc_timing_end(hc_ctx* ctx, void* stream, double* out_avg_ms, int32_t* out_launches);
/* The same, also reporting the shortest and the median launch (either pointer may be NULL). */
hc_status hc_timing_end_stats(hc_ctx* ctx, void* stream, double* out_avg_ms, double* out_min_ms,
                              double* out_median_ms, int32_t* out_launches);

/* Host-side view of the restoration kernel's launch shape (no device work; for tests and
 * profiles).  For a layer of d_kv x n_tok and a launch over n_layers (1..32) layers:
 * out_shape[6] = { feature tiles, token tiles, super-tile width in feature tiles, in token
 * tiles, workgroup slots per layer, 0 }.  When out_tiles is not NULL it receives, for every
 * layer and slot in launch order, the pair (feature tile, token tile) the slot's workgroup
 * works on, or (-1, -1) for a padding slot; out_capacity is its size in pairs (HC_ERANGE when
 * too small).  Workgroup w of a launch runs on XCD w % 8. */
hc_status hc_diag_tile_map(int32_t d_kv, int32_t n_tok, int32_t n_layers, int32_t* out_shape,
                           int32_t* out_tiles, int64_t out_capacity);

/* Matrix-pipe duty-cycle probe (measurement only; evidence for how the chip's power management
 * bounds the restoration kernel).  All compute units run bursts of bf16 matrix ops on register
 * operands, busy while (wall clock mod period_us) < duty * period_us and asleep otherwise, for
 * total_us; with half_phase != 0 every other workgroup is busy in the other half of the period
 * (so half the chip is idle at any moment).  *out_tflops = matrix-op rate inside the busy
 * windows, scaled to the whole chip.  zero_operands != 0 uses all-zero operands (no operand
 * toggling).  op_shape selects the matrix op: 0 = 32x32x16, 1 = 16x16x32 (the
 * restoration kernel's; same flop per burst).  Allocates and frees small device buffers, synchronises the
 * device. */
hc_status hc_diag_mfma_duty(double period_us, double duty, int32_t half_phase, double total_us,
                            int32_t zero_operands, int32_t op_shape, double* out_tflops);

#ifdef __cplusplus
}
#endif
#endif /* HCACHE_H */
