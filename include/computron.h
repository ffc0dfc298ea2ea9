/*
 * computron.h — C ABI of the MI355X model-swapping library.
 *
 * One GPU's share of model-parallel swapping (Computron, arXiv 2306.13835):
 * the fp16 parameters of one tensor-parallel rank of an OPT decoder live in
 * page-locked host memory (Section 3.2, last paragraph), are swapped into a
 * device arena when the model is requested and swapped out again when a
 * least-recently-used replacement policy needs the room (Section 3, demand
 * paging; Section 4, LRU).  Loads, offloads and inference run on three
 * separate streams (Section 3.2).  Beyond the paper, a load is split layer by
 * layer and every layer signals an event, so the forward pass of the same
 * model may start as soon as its first layers have landed.
 *
 * Conventions
 *   - Every function returns 0 (CTN_OK) or a negative CTN_E_* code; nothing
 *     throws across the boundary.  After CTN_E_HIP, ctn_last_hip_error()
 *     returns the HIP status that caused it.
 *   - "host" pointers are ordinary process addresses; "device" pointers are
 *     HIP device addresses.  Each argument says which it is.
 *   - The library never allocates or frees device memory: the arena, the
 *     workspace and the streams belong to the caller and must outlive the
 *     context.  It owns only host-side descriptors, its events and a few KB
 *     of pinned host memory in which it stages token ids.
 *   - A context is not thread safe; use one host thread per context.
 *   - An engine borrows its context: destroy engines before their context.
 *     "streams ... belong to the caller" applies when the caller passes
 *     streams; with none given the library creates and owns its streams.
 */
#ifndef COMPUTRON_H
#define COMPUTRON_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif
#pragma GCC visibility push(default) /* the entry points below are the library's only exports */

typedef struct ctn_ctx ctn_ctx;
typedef int32_t ctn_model;

enum {
  CTN_OK = 0,
  CTN_E_INVAL = -1,   /* bad argument: null, inconsistent description, size/shape mismatch, misalignment */
  CTN_E_TOO_BIG = -2, /* shard larger than the budget or the arena */
  CTN_E_NOMODEL = -3, /* unknown model handle */
  CTN_E_BUSY = -4,    /* no room can be made (nothing evictable) */
  CTN_E_HIP = -5,     /* a HIP call failed; see ctn_last_hip_error() */
  CTN_E_SHAPE = -6,   /* batch/seq outside what the model or the workspace allows */
  CTN_E_NOMEM = -7    /* host allocation failed / workspace too small for the library's tables */
};

enum { CTN_XFER_DMA = 0, CTN_XFER_KERNEL = 1, CTN_XFER_AUTO = 2,
       CTN_XFER_DMA_IN_KERNEL_OUT = 3, CTN_XFER_KERNEL_IN_DMA_OUT = 4, CTN_XFER_DMA_RUNS = 5 };

/* One rank's share of an OPT decoder.  layers, heads, ffn and vocab are those
 * of the whole model; the rank owns heads/tp heads, ffn/tp hidden units,
 * vocab/tp token rows.  pp > 1 (Section 5.1: models are split by tensor and by
 * pipeline parallelism): the shard is pipeline stage `stage` of pp and holds
 * the layers [stage*layers/pp, (stage+1)*layers/pp); stage 0 also holds the
 * embeddings, the last stage the final LayerNorm and its own copy of the tied
 * head matrix.  pp of 0 or 1: all layers.  Requirements: hidden % heads == 0,
 * hidden <= 16384, head size 64 or 128, heads % tp == 0, ffn % tp == 0, vocab % tp == 0,
 * (hidden/tp) % 8 == 0, (ffn/tp) % 8 == 0, 0 <= rank < tp, max_pos >= 1,
 * layers % pp == 0, 0 <= stage < pp. */
typedef struct {
  int32_t layers, hidden, ffn, heads, vocab, max_pos, tp, rank;
  int32_t pp, stage;
} ctn_model_desc;

/* One parameter tensor, fp16, C-contiguous.  host_ptr (host, also readable
 * and writable by the device: memory from ctn_host_alloc or any other
 * hipHostMalloc'ed mapping) stays the caller's and must stay valid until the
 * context is destroyed.  nbytes must equal 2*prod(shape) and be a multiple
 * of 16; host_ptr must be 16-byte aligned. */
typedef struct {
  void* host_ptr;
  uint64_t nbytes;
  int32_t ndim;      /* 1 or 2 */
  int64_t shape[2];  /* shape[1] ignored when ndim == 1 */
} ctn_param;

typedef struct {
  uint64_t hbm_budget_bytes; /* cap on the parameter bytes resident at once (arena bytes only) */
  void* arena_dev;           /* device; 256-byte aligned; holds resident shards */
  uint64_t arena_bytes;
  void* workspace_dev;       /* device; 256-byte aligned; activations + the library's tables */
  uint64_t workspace_bytes;
  void* stream_compute;      /* hipStream_t; inference kernels */
  void* stream_h2d;          /* hipStream_t; swap-in  */
  void* stream_d2h;          /* hipStream_t; swap-out */
                             /* All three NULL: the library creates and owns three streams, each on
                                its own hardware queue and confined to its own compute units
                                (copy_cus per transfer direction, the rest for inference), so copy
                                wavefronts waiting on the host link never share a compute unit with
                                the forward pass.  Otherwise all three must be given, distinct. */
  int32_t transfer_mode;     /* CTN_XFER_DMA: one hipMemcpyAsync per tensor (the paper's per-tensor
                                messages, Section 5.1); CTN_XFER_KERNEL: one copy kernel per layer
                                block, both directions; CTN_XFER_DMA_RUNS: one hipMemcpyAsync per run of
                                tensors that lie back to back on the host, both directions;
                                CTN_XFER_DMA_IN_KERNEL_OUT / CTN_XFER_KERNEL_IN_DMA_OUT: the copy kernel
                                in one direction, one DMA copy per run in the other (with
                                copy_waves_out == 0 the offloads that a miss causes take the width that
                                keeps pace with the load beside them, as under CTN_XFER_AUTO).
                                CTN_XFER_AUTO, decided per miss from the context's own record and its
                                events (never the clock): a host list in many separate pieces is loaded
                                by the copy kernel when the link's other direction is idle (the miss
                                evicts nothing and no earlier offload is still running), else by one DMA
                                copy per large run plus one narrow copy-kernel launch per block that
                                gathers its small tensors, with the victims' offloads going through the copy
                                kernel at a width that keeps the two directions at the same pace (library-
                                owned streams; on the caller's streams those offloads are DMA copies); an explicit
                                ctn_swap_out uses the copy kernel at full width; a list whose tensors
                                lie back to back on the host takes one DMA copy per run both ways */
  int32_t pipeline;          /* 0: inference waits for the whole shard (the paper's rule, Section 3.2);
                                1: inference waits layer by layer */
  int32_t copy_blocks;       /* workgroups (256 threads) of a copy kernel; 0 = library default */
  int32_t copy_cus;          /* library-owned streams only: compute units reserved per transfer
                                direction, at least 8 (one per XCD); 0 = library default */
  int32_t block_residency;   /* 0: a model is resident or not as a whole (the paper's demand paging,
                                Section 3).  1: residency per transfer block: what stays of a model
                                is a prefix of its blocks (embeddings, then layer by layer); a miss
                                evicts only as many blocks as it needs, from the tail of the least
                                recently used model, and a later use of that model reloads just the
                                missing tail while its forward pass starts on the prefix.  Every
                                block then occupies one slot of ctn_slot_bytes() in the arena. */
  int32_t discard_on_evict;  /* 0 (default, the paper's behaviour): an evicted model is copied back into
                                its host tensors (Section 3.2: offload entries).  1: inference never
                                writes parameters, so eviction only frees the device copy and the host
                                tensors, which the caller must then leave unchanged while the model is
                                registered, stay the single source; nothing crosses the link on swap-out. */
  int32_t copy_waves_out;    /* wavefronts of an offload's copy kernel (a multiple of 4 runs as workgroups of
                                256 threads, another even count as workgroups of 128, an odd count as
                                single wavefronts); 0 = 4 * copy_blocks, as for loads */
} ctn_config;

typedef struct {
  uint64_t bytes_h2d, bytes_d2h;       /* parameter bytes moved so far */
  uint64_t n_swap_in, n_swap_out;      /* completed enqueue operations */
  uint64_t n_hit, n_miss;              /* uses that found / did not find the model resident */
  uint64_t n_infer;
  uint64_t resident_bytes, peak_resident_bytes;
  uint64_t budget_bytes;
  uint64_t n_partial_miss;             /* misses that found a prefix of the model resident (block residency) */
  uint64_t n_extra_evictions;          /* eviction steps taken because no arena hole was wide enough
                                          although the budget had room (not part of the policy) */
  uint64_t n_prefetch;                 /* swap-ins started ahead of a request by ctn_engine_idle */
} ctn_stats;

/* Residency event, in the order decisions were taken (Section 3: replacement
 * on demand).  kind: 0 hit, 1 miss (victims swapped out first), 2 explicit
 * swap-out.  victims are model handles, least recently used first. */
typedef struct {
  int32_t kind;
  int32_t model;
  int32_t n_victims;
  int32_t victims[13];
} ctn_event;

/* Block-level record of the same decisions: blocks [first_block, end_block) of
 * `model` were loaded (kind 0) or evicted (kind 1) by use number `use` (index
 * into the ctn_event log).  Evictions of one use come before its load, victims
 * least recently used first. */
typedef struct {
  int32_t kind;
  int32_t model;
  int32_t first_block, end_block;
  uint64_t use;
} ctn_block_event;

/* ---- life cycle ---------------------------------------------------------- */

/* Creates a context on the current HIP device.  cfg (host) is copied. */
int ctn_create(const ctn_config* cfg, ctn_ctx** out);
/* Synchronises the three streams, destroys events; frees no caller memory. */
int ctn_destroy(ctn_ctx* ctx);

/* Page-locked, device-mapped host memory for parameters (Section 3.2: the
 * host copy stays pinned so no staging copy is needed).  *out is a host
 * pointer that kernels may also dereference.  Freed by ctn_host_free only. */
int ctn_host_alloc(uint64_t nbytes, void** out);
int ctn_host_free(void* p);

/* Registers one rank's parameter list (Section 3.1: every worker manages its
 * shard of every co-located model).  params (host array of n entries) lists
 * the tensors in forward order:
 *   embed_tokens[vocab/tp, hidden], embed_positions[max_pos+2, hidden],
 *   per layer: ln1.w ln1.b q.w[hidden/tp, hidden] q.b k.w k.b v.w v.b
 *              o.w[hidden, hidden/tp] o.b[hidden] ln2.w ln2.b
 *              fc1.w[ffn/tp, hidden] fc1.b fc2.w[hidden, ffn/tp] fc2.b[hidden],
 *   final_ln.w, final_ln.b                       (n == 16*layers + 4).
 * A pipeline stage (desc->pp > 1) lists: the two embeddings only on stage 0;
 * its own layers; final_ln.w, final_ln.b and then lm_head[vocab/tp, hidden]
 * (the stage's copy of the tied head matrix) only on the last stage.
 * Weight matrices are [out, in] row major.  hbm_budget_bytes is the manager
 * wide budget: 0 keeps the context's value, any other value must equal it.
 * The model starts swapped out.  Errors: CTN_E_INVAL, CTN_E_TOO_BIG. */
int ctn_register_model(ctn_ctx* ctx, const ctn_model_desc* desc, const ctn_param* params,
                       size_t n, uint64_t hbm_budget_bytes, ctn_model* out);

/* ---- swapping (Section 3.2: load / offload entries, asynchronous) --------- */

/* Counts as a use.  If the model is not resident, swaps out least recently
 * used models until it fits, then enqueues its load on the h2d stream, layer
 * block by layer block in forward order, one event per block.  Returns
 * without waiting.  Resident model: success, nothing moved. */
int ctn_swap_in(ctn_ctx* ctx, ctn_model m);
/* Enqueues the copy of every tensor back to its host buffer on the d2h
 * stream (after the model's last inference, on the device), then releases its
 * arena range.  Non-resident model: success, nothing moved. */
int ctn_swap_out(ctn_ctx* ctx, ctn_model m);
/* Blocks the host until the model's pending load or offload has finished. */
int ctn_wait(ctn_ctx* ctx, ctn_model m);
/* Blocks the host until all three streams are idle. */
int ctn_sync(ctn_ctx* ctx);

/* ---- inference ------------------------------------------------------------ */

/* Forward pass of the rank's shard on token ids (host, int32 [batch, seq],
 * values in [0, vocab)): logits fp32 [batch, seq, vocab/tp].  Row-parallel
 * products are this rank's partial sums (the cross-rank reduction is the
 * identity on one GPU).  Counts as a use; a non-resident model is swapped in
 * first (demand paging, Section 3).  token_ids_host (ordinary host memory) is
 * copied into a pinned staging buffer of the context before the call returns,
 * in every case, so the caller may reuse it at once.  logits_out is a device pointer when
 * out_is_device != 0 (the call returns with the work enqueued on the compute
 * stream), else pinned or ordinary host memory (the call returns after the
 * logits have arrived).  Errors: CTN_E_SHAPE when batch or seq is not positive,
 * seq > max_pos, batch > 65535, batch*seq > 2^24 or the workspace cannot hold
 * batch*seq tokens (see ctn_workspace_bytes); CTN_E_INVAL for a token id outside
 * [0, vocab).  Nothing is enqueued and no residency decision is taken when
 * either is returned. */
int ctn_infer(ctn_ctx* ctx, ctn_model m, const int32_t* token_ids_host, int32_t batch, int32_t seq,
              void* logits_out, int32_t out_is_device);
/* The same for any pipeline stage.  Stage 0 starts from token_ids_host
 * (hidden_in must be NULL); later stages start from hidden_in, the residual
 * stream fp32 [batch, seq, hidden] the previous stage emitted (device pointer
 * when in_is_device != 0, else host; token_ids_host is ignored).  out receives
 * fp32 [batch, seq, hidden] (the residual stream after the stage's last
 * layer) or, on the last stage, the logits fp32 [batch, seq, vocab/tp].
 * ctn_infer(m, ids, ...) is ctn_infer_stage(m, ids, NULL, 0, ...). */
int ctn_infer_stage(ctn_ctx* ctx, ctn_model m, const int32_t* token_ids_host, const void* hidden_in,
                    int32_t in_is_device, int32_t batch, int32_t seq, void* out, int32_t out_is_device);

/* Workspace bytes a context needs for models of this description at up to
 * max_tokens = batch*seq tokens per inference and n_models registrations.  Never decreases as
 * max_tokens grows: a workspace of this size serves every smaller batch as well. */
uint64_t ctn_workspace_bytes(const ctn_model_desc* desc, int64_t max_tokens, int32_t n_models);
/* Arena bytes one shard of this description occupies (tensors padded to 256 B). */
uint64_t ctn_arena_bytes(const ctn_model_desc* desc);
/* Block residency: bytes of the arena slot each of the shard's layers+1 transfer
 * blocks occupies (the widest block, padded), so a shard takes (layers+1) slots. */
uint64_t ctn_slot_bytes(const ctn_model_desc* desc);

/* ---- introspection -------------------------------------------------------- */

/* *out = 1 when every block of the model is resident (or on its way in). */
int ctn_is_resident(ctn_ctx* ctx, ctn_model m, int32_t* out);
/* Number of resident transfer blocks (a prefix) and the model's block count. */
int ctn_resident_blocks(ctn_ctx* ctx, ctn_model m, int32_t* resident, int32_t* total);
int ctn_get_stats(ctn_ctx* ctx, ctn_stats* out);
/* Copies up to cap events starting at index first into out (host); *n_out
 * receives the number copied, *total the number recorded so far. */
int ctn_get_events(ctn_ctx* ctx, uint64_t first, ctn_event* out, uint64_t cap, uint64_t* n_out,
                   uint64_t* total);
int ctn_get_block_events(ctn_ctx* ctx, uint64_t first, ctn_block_event* out, uint64_t cap, uint64_t* n_out,
                         uint64_t* total);
/* Device-timeline duration (ms) of the model's last completed load and
 * offload, and the start-to-event time of each of its layer blocks
 * (block_ms: host array of cap floats or NULL; blocks = layers + 1:
 * embeddings with the final LayerNorm, then each layer).  Blocks until they have finished. */
int ctn_last_swap_ms(ctn_ctx* ctx, ctn_model m, float* in_ms, float* out_ms, float* block_ms,
                     int32_t cap, int32_t* n_blocks);
/* The three streams in use (hipStream_t), the library's own or the caller's. */
int ctn_get_streams(ctn_ctx* ctx, void** compute, void** h2d, void** d2h);
/* Library-owned streams only: replay captured HIP graphs for inferences on completely resident
 * models while the link is idle; 0 (the default: replay measured no faster than direct launches
 * on ROCm 7.2) launches every kernel directly. */
int ctn_set_graphs(ctn_ctx* ctx, int32_t enable);
/* Switches ctn_config.discard_on_evict between operations (evictions already decided keep their mode). */
int ctn_set_discard(ctn_ctx* ctx, int32_t enable);
/* Changes transfer mode / pipelining / copy-kernel width between operations. */
int ctn_set_mode(ctn_ctx* ctx, int32_t transfer_mode, int32_t pipeline, int32_t copy_blocks);
/* Width of the copy kernel between operations: workgroups (of 256 threads) for loads, wavefronts for
 * offloads; 0 = library default / the same width as loads. */
int ctn_set_copy_width(ctn_ctx* ctx, int32_t blocks_in, int32_t waves_out);
/* HIP status behind the last CTN_E_HIP of this context (ctx == NULL: of calls that take no context). */
int ctn_last_hip_error(ctn_ctx* ctx);
const char* ctn_strerror(int code);

/* ---- serving engine (Section 3.1: per-model request queues, oldest first;
 *      Section 5.2: maximum batch size) ----------------------------------------- */

typedef struct ctn_engine ctn_engine;

/* One dispatched batch of a replay: requests[offset .. offset+count) of the flat
 * request array (indices into the trace, oldest first), all of `model`. */
typedef struct {
  double start, finish;
  int32_t model, count, miss, reserved;
  uint64_t offset;
} ctn_batch_record;

/* An engine over a context: one FIFO queue per registered model, batches of at
 * most max_batch requests, every request exactly seq tokens long. */
int ctn_engine_create(ctn_ctx* ctx, int32_t max_batch, int32_t seq, ctn_engine** out);
int ctn_engine_destroy(ctn_engine* eng);
/* Queues one request: ids (host, int32[seq], values in [0, vocab)) are copied;
 * timestamp is the caller's clock (seconds).  *request_id counts from 0. */
int ctn_engine_submit(ctn_engine* eng, ctn_model m, const int32_t* ids_host, double timestamp,
                      int64_t* request_id);
/* Dispatches one batch: the queue whose oldest request is oldest, up to
 * max_batch of its requests, one ctn_infer (a use for the LRU policy; swaps as
 * needed).  logits_out (device, fp32 [max_batch, seq, vocab/tp]) receives the
 * batch's logits, request k of the batch in row k; the call returns with the
 * work enqueued on the compute stream.  served_ids (host, cap >= max_batch)
 * receives the request ids; *n_served == 0 when nothing is queued. */
int ctn_engine_step(ctn_engine* eng, void* logits_out, int64_t* served_ids, int32_t cap, int32_t* n_served,
                    ctn_model* model, int32_t* was_miss);
int ctn_engine_pending(ctn_engine* eng, int64_t* n);

/* The two-lane engine (Section 3.2: load entries are asynchronous, so a batch
 * of one model need not wait for the load of another).  Lane 0 runs batches of completely loaded
 * models, one at a time; lane 1 takes one miss at a time, the model's swap-in
 * followed, block by block, by its batch; a model whose miss is in flight is
 * not dispatched again until that batch has completed.  Needs a context with
 * library-owned streams and twice the workspace of ctn_workspace_bytes() (each
 * lane works in its own half; destroying the engine gives the context its whole
 * workspace back).  ctn_engine_step is not available on it. */
int ctn_engine_create_async(ctn_ctx* ctx, int32_t max_batch, int32_t seq, ctn_engine** out);
/* Dispatches at most one batch: the non-empty queues are scanned oldest head
 * first and the first whose lane is free and whose model is not loading goes.
 * logits_out[lane] (device, fp32 [max_batch, seq, vocab/tp], one buffer per
 * lane) receives the batch's logits; the call returns with the work enqueued.
 * *n_served == 0 when nothing can be dispatched now (queues empty, lanes busy
 * or models loading).  *lane tells where the batch runs (0 hit lane, 1 load lane;
 * a model that ctn_engine_idle started loading and that is still arriving also
 * takes the load lane, with *was_miss == 0). */
int ctn_engine_dispatch(ctn_engine* eng, void* const logits_out[2], int64_t* served_ids, int32_t cap,
                        int32_t* n_served, ctn_model* model, int32_t* was_miss, int32_t* lane);
/* busy[l] = 1 while the batch last dispatched on lane l has not completed
 * (host array of 2).  Does not block. */
int ctn_engine_lanes(ctn_engine* eng, int32_t* busy);
/* Loading ahead (the paper's closing section: speculative loads for request
 * streams with structure).  The engine keeps a first-order transition table
 * over its dispatches; after a dispatch of model a it predicts the model that
 * most often followed a (ties: lowest handle) if that was seen at least
 * min_count times and is at least min_share_percent per cent of the
 * transitions out of a.  enable == 0 switches it off (the default). */
int ctn_engine_set_prefetch(ctn_engine* eng, int32_t enable, int32_t min_count, int32_t min_share_percent);
/* To be called when the caller has nothing to submit.  If no request is
 * queued, loading ahead is on and the predicted model is not completely
 * resident, it is swapped in (an ordinary ctn_swap_in: asynchronous, a use
 * for the replacement policy, victims evicted as needed).  *loaded receives
 * that model's handle, -1 when nothing was done. */
int ctn_engine_idle(ctn_engine* eng, ctn_model* loaded);
/* ---- single operations (each enqueues on `stream`, a hipStream_t; all data
 *      pointers are device pointers unless stated).  The kernels read and write
 *      rows in 16-byte pieces: matrices and activations must start on a 16-byte
 *      boundary (vectors of gains and biases on an 8-byte one, the bias of a
 *      product on a 2-byte one, ids and fp32 outputs of a product on a 4-byte
 *      one); CTN_E_INVAL otherwise, and for shapes a kernel does not cover. ---- */

enum { CTN_EPI_BIAS_F16 = 0,       /* out fp16 [M,N]  = A W^T + bias            */
       CTN_EPI_BIAS_RELU_F16 = 1,  /* out fp16 [M,N]  = max(0, A W^T + bias)    */
       CTN_EPI_BIAS_RESID_F32 = 2, /* out fp32 [M,N] += A W^T + bias (in place) */
       CTN_EPI_F32 = 3 };          /* out fp32 [M,N]  = A W^T (bias ignored)    */

/* Copy kernel over one byte range (16-byte multiple, 16-byte aligned ends).
 * src/dst may each be device memory or device-mapped pinned host memory: the
 * same kernel serves swap-in and swap-out (Section 3.2).  blocks = workgroups. */
int ctn_op_copy(void* dst, const void* src, uint64_t nbytes, int32_t blocks, void* stream);
/* hipMemcpyAsync of one range (the DMA engine path), for link-peak measurements. */
int ctn_op_dma(void* dst, const void* src, uint64_t nbytes, void* stream);
/* x fp32 [M,hidden] = token row (zero if id outside [rank*vocab_local,
 * (rank+1)*vocab_local)) + position row (m mod seq) + 2.  ids int32 [M].
 * hidden % 8 == 0. */
int ctn_op_embed(const int32_t* ids, const void* tok_f16, const void* pos_f16, float* x, int32_t M,
                 int32_t seq, int32_t hidden, int32_t vocab_local, int32_t rank, void* stream);
/* out fp16 [rows,hidden] = LayerNorm(x fp32; gain, bias fp16), biased variance, eps 1e-5.
 * hidden % 4 == 0, hidden <= 16384. */
int ctn_op_layernorm(const float* x, const void* gain_f16, const void* bias_f16, void* out_f16,
                     int32_t rows, int32_t hidden, void* stream);
/* C = A[M,K] (fp16) times W[N,K]^T (fp16), fp32 accumulation on the matrix
 * cores, then the chosen epilogue.  K % 8 == 0. */
int ctn_op_gemm(const void* A_f16, const void* W_f16, const void* bias_f16, void* out, int32_t M,
                int32_t N, int32_t K, int32_t epilogue, void* stream);
/* The same product with a device scratch buffer (16-byte aligned; may be NULL): products with
 * M <= 256 (and larger ones with few tiles and K >= 2048, or, in the columns of a thinly filled
 * last round of tiles, any product with K >= 2048) may then cut K into slices computed by
 * separate workgroups, whose fp32 partial tiles are added in a fixed order, so the result does
 * not depend on timing.  ctn_infer does the same
 * with a slice of its workspace. */
int ctn_op_gemm_ws(const void* A_f16, const void* W_f16, const void* bias_f16, void* out, int32_t M,
                   int32_t N, int32_t K, int32_t epilogue, void* workspace, uint64_t workspace_bytes,
                   void* stream);
/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): ctn_op_gemm_ws with the scratch buffer taken from a static device
 * array of ctn_static_scratch_bytes() (64 MiB) that every GPU the library runs on holds until the process
 * ends.  Calls no hipMalloc / hipFree and no allocating routine.  The product may be cut into up to 16
 * K slices (M <= 256) or 4 (larger M); shapes whose slices would not fit, 4*M*N*16 (M <= 256) or 4*M*N*4
 * bytes beyond the array's size, return CTN_E_TOO_BIG.  Results equal ctn_op_gemm_ws with a workspace of
 * the same size, bit for bit.  All calls on one GPU share the array (every slice is written before it is
 * read, so stale contents do no harm): two calls that overlap in time on one GPU, on different streams
 * or from different threads, race; calls on one stream are ordered. */
int ctn_op_gemm_static(const void* A_f16, const void* W_f16, const void* bias_f16, void* out, int32_t M,
                       int32_t N, int32_t K, int32_t epilogue, void* stream);
uint64_t ctn_static_scratch_bytes(void);
/* Causal self-attention of every (batch, head): qkv fp16 [batch*seq, 3*heads*d]
 * holds q | k | v side by side; out fp16 [batch*seq, heads*d]
 * = softmax_causal((q d^-1/2) k^T) v.  d is 64 or 128; batch and heads at most 65535 each. */
int ctn_op_attention(const void* qkv_f16, void* out_f16, int32_t batch, int32_t seq, int32_t heads,
                     int32_t head_dim, void* stream);

#pragma GCC visibility pop
#ifdef __cplusplus
}
#endif
#endif
