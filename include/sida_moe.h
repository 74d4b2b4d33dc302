/* sida_moe.h — C ABI of the SiDA-MoE layer hot path for AMD MI355X (gfx950).
 *
 * The library serves one sparse Mixture-of-Experts layer at a time the way the paper's inference
 * thread does (Section 3.1; Algorithm 1, left column): the expert id and the scaling factor
 * alpha of every token come from a table that was built ahead of time (the "hash table" H[l][s]),
 * routers take no part, only experts that have tokens are invoked (Section 2.3), and only the
 * experts a batch activates are kept in GPU memory, in a pool of S equal-sized slots that is
 * filled from host memory and replaced first-in-first-out (Section 3.1, Section 4.3).
 *
 * Layer output (Section 2.1, Eq. 1 with the Switch top-1 selection):
 *     y[t,:] = alpha[t] * W_out[k] * relu(W_in[k] * x[t,:]),     k = expert_ids[t]
 *
 * Conventions
 *  - "host" pointers are ordinary process memory; "device" pointers are HIP device memory of the
 *    current device.  The library never allocates or frees device memory: x, y, ids, alpha, the
 *    slot pool and the workspace are the caller's, and so are the pinned host weight blocks.
 *  - Streams are passed as raw hipStream_t values cast to void* (NULL = the null stream).
 *  - bf16 = bfloat16 (upper half of an IEEE fp32).  All matrices are row-major.
 *  - One expert is ONE contiguous host block of sida_expert_bytes() bytes:
 *        W_in  bf16 [d_ff, d_model]   (row j = weights of hidden unit j), immediately followed by
 *        W_out bf16 [d_model, d_ff].
 *    Slot s of the pool is the byte range [s*expert_bytes, (s+1)*expert_bytes).  Inside a slot
 *    the library keeps the two matrices in the order its matrix-core kernels read them
 *    (sida_slot_offset): the prefetch re-orders an expert on its way into the slot, so a slot is
 *    NOT a byte copy of the host block and is only ever filled through sida_expert_prefetch (or
 *    the forward calls that prefetch).
 *  - Every function returns SIDA_OK (0) or a negative sida_status.  Arguments and state are
 *    checked before anything else: on SIDA_EINVAL, SIDA_ENOSPC, SIDA_ESTATE, SIDA_ENOMEM,
 *    SIDA_EAGAIN and SIDA_ECLOSED nothing has been enqueued and no bookkeeping has changed.
 *    SIDA_EHIP means a HIP call failed part-way: launches and copies enqueued before it stay
 *    enqueued and the waves they belong to count as prefetched / forwarded; drain the streams and
 *    call sida_pool_reset() before using the context again.  Faults of work that was already
 *    enqueued show up at the caller's next stream synchronisation, as with any HIP work.
 *  - A context is not thread-safe (the hash-table queue calls excepted); use one per serving thread.  All compute of one context must
 *    be enqueued on one stream, all copies on one (other) stream.
 *  - Limits: 1 <= E <= SIDA_MAX_E; d_model and d_ff multiples of 128, 128 .. 4096; 1 <= W <= S;
 *    max_T * max(d_model, d_ff) * 2 < 2^31 (rows are addressed with 32-bit byte offsets).
 */
#ifndef SIDA_MOE_H
#define SIDA_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SIDA_MAX_E 256

typedef enum sida_status {
    SIDA_OK = 0,
    SIDA_EINVAL = -1,   /* null pointer, bad shape, expert id outside [0,E), bad wave index   */
    SIDA_ENOSPC = -2,   /* workspace or pool smaller than required                            */
    SIDA_ESTATE = -3,   /* pool / host weights not bound, stale plan, calls out of wave order  */
    SIDA_EHIP = -4,     /* a HIP call failed; see sida_last_hip_error()                        */
    SIDA_ENOMEM = -5,   /* host allocation failed                                              */
    SIDA_EAGAIN = -6,   /* sida_queue_pop_plan: no hash table arrived within the timeout       */
    SIDA_ECLOSED = -7   /* hash-table queue closed (and, for a pop, drained)                   */
} sida_status;

/* Replacement policy of the slot pool.  The paper uses first-in-first-out and notes that other
 * strategies could be effective too (footnote of Section 4.3). */
enum { SIDA_POLICY_FIFO = 0,    /* overwrite the oldest load; a hit does not renew an age (default) */
       SIDA_POLICY_LRU = 1,     /* overwrite the expert loaded or hit longest ago                   */
       SIDA_POLICY_BELADY = 2   /* overwrite the expert whose next use is farthest in the known
                                   future (rest of the layer, then the caller's look-ahead);
                                   ties go to the oldest load                                       */ };
#define SIDA_QUEUE_CAPACITY 256 /* hash tables the queue holds at most */

typedef struct sida_ctx sida_ctx; /* opaque: host bookkeeping and HIP events only */

typedef struct sida_config {
    int32_t L;        /* MoE layers sharing the pool                                         */
    int32_t E;        /* experts per layer                                                   */
    int32_t d_model;  /* token width d                                                       */
    int32_t d_ff;     /* hidden width F of an expert                                         */
    int32_t S;        /* expert slots in the pool (the GPU memory budget of Section 3.1)     */
    int32_t W;        /* most experts computed together as one wave, 1..S                    */
    int32_t max_T;    /* most tokens per layer call                                          */
} sida_config;

/* Residency plan of one layer for one batch: the outcome of Algorithm 1's inference-thread loop
 * (every token's expert is checked and moved to the GPU when it is not there) under the FIFO budget.  Plain data,
 * owned by the caller, filled by sida_moe_plan().  Arrays indexed by expert id hold -1 for
 * experts without tokens (they are never loaded nor invoked).  Waves carry a global index that
 * counts up over the life of the pool; a layer's waves are first_wave .. first_wave+n_waves-1. */
typedef struct sida_plan {
    int32_t layer, T, E;
    int32_t n_active;                      /* experts with at least one token                        */
    int32_t n_waves;                       /* 0 iff T == 0                                           */
    int32_t first_wave;                    /* global index of the layer's first wave, -1 if none     */
    uint32_t epoch;                        /* pool generation the plan belongs to (see pool_reset)   */
    int32_t n_miss;                        /* experts that have to be copied host -> pool            */
    int32_t counts[SIDA_MAX_E];            /* tokens per expert                                      */
    int32_t offsets[SIDA_MAX_E + 1];       /* exclusive prefix sum of counts; offsets[E] == T        */
    int32_t order[SIDA_MAX_E];             /* activated experts in order of first appearance         */
    int32_t slot[SIDA_MAX_E];              /* pool slot holding the expert while its wave computes   */
    int32_t wave[SIDA_MAX_E];              /* global wave the expert is computed in                  */
    int32_t hit[SIDA_MAX_E];               /* 1: already resident, 0: must be copied                 */
    int32_t evicted_key[SIDA_MAX_E];       /* layer*E+e overwritten by this expert's copy, -1 none   */
    int32_t wave_dep[SIDA_MAX_E];          /* per local wave: global wave whose compute must finish
                                              before this wave's copies may start, -1 if none       */
} sida_plan;

/* Byte offsets of the regions inside the caller's workspace for a call with T tokens (tests and
 * profilers read intermediates through these). */
typedef struct sida_ws_layout {
    size_t counts;      /* int32 [E]                    tokens per expert                     */
    size_t offsets;     /* int32 [E+1]                  exclusive prefix sum                  */
    size_t block_hist;  /* int32 [n_blocks*E]           per-block histograms, then bases      */
    size_t perm;        /* int32 [T]   perm[r] = t      stable order by (expert, token)       */
    size_t inv;         /* int32 [T]   inv[t]  = r                                            */
    size_t x_perm;      /* bf16  [T, d_model]           x rows in perm order                  */
    size_t h;           /* bf16  [T, d_ff]              relu(x_perm W_in^T), perm order       */
    size_t y_perm;      /* bf16  [T, d_model]           expert outputs, perm order            */
    size_t tiles;       /* int32 [4 * (T/64 + E + 1)]   token-tile descriptors of the grouped FFN */
    size_t sink;        /* 64 KiB scratch: absorbs the grouped FFN's stores of rows past a tile's end */
    size_t gate_perm;   /* fp32  [T]   gate_perm[r] = alpha[perm[r]]   (fused path only)      */
    size_t total;       /* bytes needed                                                       */
} sida_ws_layout;

/* ---- context ------------------------------------------------------------------------------ */

/* Validates cfg and creates a context with an empty pool.  Touches no GPU. */
int sida_create(const sida_config *cfg, sida_ctx **out);
/* Destroys the context and its HIP events.  Does not synchronise: the caller must have drained
 * the streams first.  NULL is allowed. */
void sida_destroy(sida_ctx *ctx);
const char *sida_strerror(int code);
/* hipError_t (as int) of the HIP call behind the last SIDA_EHIP of this context, else 0. */
int sida_last_hip_error(const sida_ctx *ctx);

/* 4 * d_model * d_ff: W_in and W_out of one expert in bf16 (two d_model x d_ff matrices, the
 * per-expert parameter count behind Table 2 of Section 2.2). */
size_t sida_expert_bytes(const sida_ctx *ctx);
/* Where the slot keeps element [row, col] of an expert's matrix (which = 0: W_in [d_ff, d_model],
 * 1: W_out [d_model, d_ff]), in bytes from the start of the slot; (size_t)-1 on bad arguments.
 * A matrix [R, K] is stored in stripes of 32 rows; inside a stripe the 16-byte pieces (8
 * consecutive K values of one row) are ordered piece-major, row-minor, so that the 32 rows x 16
 * K values one 32x32x16 matrix-core instruction takes as an operand are 1 KiB of consecutive
 * memory:  offset = ((row/32) * (K/8) + col/8) * 512 + (row%32) * 16 + (col%8) * 2.
 * For tests and tools that inspect the pool. */
size_t sida_slot_offset(const sida_ctx *ctx, int32_t which, int32_t row, int32_t col);
/* Workspace bytes a layer call with T tokens needs (0 on bad arguments). */
size_t sida_workspace_bytes(const sida_ctx *ctx, int32_t T);
int sida_workspace_layout(const sida_ctx *ctx, int32_t T, sida_ws_layout *out);

/* pool_dev: device memory, 256-byte aligned, bytes >= S * expert_bytes, owned by the caller and
 * kept alive while the context uses it. */
int sida_bind_pool(sida_ctx *ctx, void *pool_dev, size_t bytes);
/* host_blocks: host array of L*E pointers, entry layer*E+e -> that expert's block in PINNED host
 * memory (pageable memory works but makes the copies synchronous and rules out the copy kernel).  The pointer table is copied;
 * the blocks stay the caller's and must outlive every prefetch that reads them. */
int sida_bind_host_weights(sida_ctx *ctx, const void *const *host_blocks);
/* Creates the two streams a context's work is enqueued on (default priority, non-blocking with
 * respect to the null stream), with the chip's compute units divided between them: copy_stream
 * may use copy_cus of them (a multiple of 8, taken evenly from the XCDs; at most half), the
 * compute stream all the others, and the grouped GEMMs size their persistent grids to the
 * compute units of the stream they run on.  This keeps the copy kernel of SIDA_PREFETCH_KERNEL off
 * the compute units of the GEMMs: a GEMM that shares a compute unit with workgroups waiting on
 * host-link reads runs 2-3 x slower (measured), because vector memory returns of a compute unit
 * come back in order.  copy_cus = 0: two plain streams.  Any other streams may be passed to the
 * forward calls instead.  Destroy the streams after the context's work has drained. */
int sida_streams_create(int32_t copy_cus, void **compute_stream, void **copy_stream);
int sida_streams_destroy(void *compute_stream, void *copy_stream);

/* How sida_expert_prefetch moves an expert into its slot.
 *   SIDA_PREFETCH_COPY_ENGINE  one hipMemcpyAsync per expert (works with pageable host memory too),
 *                              then one kernel per wave that re-orders the copied slots in place;
 *   SIDA_PREFETCH_KERNEL       one copy kernel per wave that reads the pinned blocks over the host
 *                              link itself and writes the slot order directly: no per-expert cost
 *                              (57 GB/s against 45 GB/s measured with 9.4 MB experts); needs every
 *                              bound block in pinned memory, SIDA_ESTATE otherwise (bind the
 *                              weights first);
 *   SIDA_PREFETCH_AUTO         the kernel when every bound block is pinned, else the copy engine
 *                              (default). */
enum { SIDA_PREFETCH_AUTO = 0, SIDA_PREFETCH_COPY_ENGINE = 1, SIDA_PREFETCH_KERNEL = 2 };
int sida_set_prefetch_mode(sida_ctx *ctx, int32_t mode);

/* Forgets every resident expert: empty pool, FIFO cursor 0, wave counter 0, new epoch (plans
 * made before the reset are stale).  The caller must have drained both streams. */
int sida_pool_reset(sida_ctx *ctx);
/* Inspection: slot_key[S] (layer*E+e or -1 per slot), FIFO cursor, next global wave index.  Any
 * output pointer may be NULL. */
int sida_pool_state(const sida_ctx *ctx, int32_t *slot_key, int32_t *cursor, int32_t *next_wave);

/* ---- the three calls of the method --------------------------------------------------------- */

/* moe_plan(expert_ids) -> residency plan.  Algorithm 1, inference thread: walks the tokens of
 * `layer` in order, checks each token's expert against the pool and schedules a load for every
 * expert that is not resident; slots are reused first-in-first-out (Section 3.1), a hit does not
 * renew an expert's age, and the budget is shared by all layers.  When a layer activates more
 * experts than one wave may hold, it is cut into waves of at most W experts.
 * Host only, integers only, synchronous.  Updates the pool BOOKKEEPING (which key each slot will
 * hold once the plan's copies ran); plans must be made in the order their layers will run.
 * ids_host: host int32 [T], 0 <= T <= max_T.  An id outside [0,E) -> SIDA_EINVAL, state unchanged. */
int sida_moe_plan(sida_ctx *ctx, int32_t layer, const int32_t *ids_host, int32_t T, sida_plan *out);

/* As sida_moe_plan, with the future the hash-table queue makes known (Section 3.1: tables are
 * built ahead of the inference thread).  future_keys: host int32 [n_future], keys layer*E+e in
 * the order they will be needed after this layer (duplicates allowed, the first occurrence
 * counts).  Only SIDA_POLICY_BELADY looks at it; with no future it degenerates to "oldest load
 * among the experts this layer does not need any more".  A key outside [0, L*E) -> SIDA_EINVAL. */
int sida_moe_plan_lookahead(sida_ctx *ctx, int32_t layer, const int32_t *ids_host, int32_t T,
                            const int32_t *future_keys, int64_t n_future, sida_plan *out);
/* Chooses the replacement policy and how many queued batches sida_queue_pop_plan may look ahead
 * at (0..SIDA_QUEUE_CAPACITY).  Only while the pool is empty (after sida_create or
 * sida_pool_reset), SIDA_ESTATE otherwise.  All policies fill empty slots first and never
 * overwrite a slot of the wave being assembled. */
int sida_set_policy(sida_ctx *ctx, int32_t policy, int32_t lookahead_batches);

/* ---- the hash-table queue between the two threads of Algorithm 1 (Section 3.1) --------------
 * The hash-building thread pushes one table per batch (the expert ids of every MoE layer); the
 * inference thread pops them in arrival order and gets the batch's residency plans, each layer
 * planned with the later layers of the batch and the queued batches behind it as its future.
 * These four calls are safe to use from two threads (one pushing, one popping); every other
 * call of a context belongs to the inference thread. */
/* ids_host: host int32 [L, T] row-major, copied.  tag: returned by the pop, for the caller to
 * find the batch's device buffers.  SIDA_ENOSPC when SIDA_QUEUE_CAPACITY tables wait already,
 * SIDA_ECLOSED after sida_queue_close, SIDA_EINVAL for an id outside [0,E) (nothing queued). */
int sida_queue_push(sida_ctx *ctx, int64_t tag, const int32_t *ids_host, int32_t T);
/* No more tables will come: pops drain the queue, then return SIDA_ECLOSED. */
int sida_queue_close(sida_ctx *ctx);
/* Tables waiting (>= 0), or a negative status. */
int sida_queue_size(sida_ctx *ctx);
/* Waits up to timeout_ms for a table (Section 3.1: the inference thread idles while its table is
 * missing), removes
 * the oldest one and plans its L layers in order, exactly as L calls of sida_moe_plan_lookahead
 * would: plans[L] (caller's array) are then run with sida_run_layers.  tag / T may be NULL.
 * SIDA_EAGAIN on timeout, SIDA_ECLOSED when closed and empty; the pool bookkeeping is untouched
 * in both cases. */
int sida_queue_pop_plan(sida_ctx *ctx, int32_t timeout_ms, int64_t *tag, int32_t *T, sida_plan *plans);

/* expert_prefetch(slot_table, host_weights, stream): enqueues, on copy_stream, the host -> pool
 * copies of the experts that local wave `wave` of `plan` misses (one copy of expert_bytes each),
 * after making copy_stream wait for the compute of wave_dep[wave] — the last wave that read a
 * slot about to be overwritten.  This is the step of Section 3.1 that loads the activated experts ahead of
 * the forward pass, overlapped with the previous compute.
 * Waves must be prefetched in global order; a wave that was already prefetched is a no-op (0).
 * SIDA_ESTATE if an earlier wave has not been prefetched yet, or if the forward call of
 * wave_dep[wave] has not been enqueued yet (the wait could not be expressed). */
int sida_expert_prefetch(sida_ctx *ctx, const sida_plan *plan, int32_t wave, void *copy_stream);

/* moe_layer_forward(x, expert_ids, gate_w, slot_table) -> y.  Eq. 1 of Section 2.1 for the T
 * tokens of plan->layer, evaluated as: stable counting sort of the tokens by expert id and
 * gather of their rows; per wave, wait for its copies, then the grouped expert FFN
 * (W_in GEMM, ReLU, W_out GEMM on bf16 MFMA, fp32 accumulate, experts addressed through the
 * plan's slot table); gate-weighted scatter back to token order.
 *   x_dev     bf16 [T, d_model]    device, read
 *   ids_dev   int32 [T]            device, read; must equal the ids the plan was made from (not
 *                                  checked unless SIDA_DEBUG_CHECK_IDS is on)
 *   alpha_dev fp32 [T]             device, read; the per-token scaling factor (gate value)
 *   y_dev     bf16 [T, d_model]    device, written
 *   workspace_dev                  device, >= sida_workspace_bytes(T), 256-byte aligned, scratch
 * Everything is enqueued on compute_stream; waves that were not prefetched yet are prefetched by
 * this call on copy_stream (one wave ahead of the compute where wave_dep allows).  Layers must
 * be forwarded in the order they were planned.  Asynchronous. */
int sida_moe_layer_forward(sida_ctx *ctx, const sida_plan *plan, const void *x_dev,
                           const int32_t *ids_dev, const float *alpha_dev, void *y_dev,
                           void *workspace_dev, size_t workspace_bytes, void *compute_stream,
                           void *copy_stream);

/* Experts per token, 1..SIDA_MAX_TOP_K (default 1 = Switch routing).  Eq. 1 of Section 2.1 with a
 * selected set of k experts: y[t,:] = sum_{j<k} alpha[t,j] * f_{ids[t,j]}(x[t,:]); the paper
 * evaluates with the hash function's top-3 experts on two of its datasets (Section 4, hyperparameters;
 * top-3 hit rates in Section 4.6).
 * With k > 1 every "T" of the plan, forward and stage calls counts (token, expert) PAIRS:
 * ids and alpha are [tokens, k] row-major (T = tokens*k entries, T <= max_T, T % k == 0,
 * SIDA_EINVAL otherwise), x and y keep one row per token (T/k rows).  The pairs are sorted and
 * run through the grouped FFN like tokens; the combine adds a token's k rows in fp32 in the order
 * j = 0..k-1 and rounds once.  A token may name the same expert more than once.
 * May be changed between layer calls; plans made before stay valid (they only count ids). */
#define SIDA_MAX_TOP_K 8
int sida_set_top_k(sida_ctx *ctx, int32_t k);

/* Folds the permute-gather into the first GEMM's token-row loads (rows are read from x through
 * the sort's index, x_perm is never written) and the gate-weighted scatter-combine into the second
 * GEMM's result stores (with top-1 routing every y row is written exactly once, by the tile that
 * holds its token; y_perm is never written).  Same arithmetic, bit-identical y; two launches and
 * about two thirds of the dispatch/combine HBM traffic less per layer.  With more than one expert
 * per token only the gather is folded in (a y row is then a sum over several tiles).  Affects
 * sida_moe_layer_forward / sida_run_layers only; the single-stage calls keep the separate passes.
 * On by default; switching it off brings the separate gather and combine passes (and the x_perm /
 * y_perm intermediates in the workspace) back.  May be switched between layer calls. */
int sida_set_fusion(sida_ctx *ctx, int32_t on);

/* Debug switches, off by default (any combination; 0 switches all off and clears a latched mismatch).
 *   SIDA_DEBUG_CHECK_IDS     sida_moe_layer_forward trusts that ids_dev holds the ids the plan was
 *                            made from (a mismatch would compute with slots and tiles that do not
 *                            belong to the rows).  With this switch every layer call also compares
 *                            the per-expert token counts its sort found on the device with the
 *                            plan's; a difference is latched, and from the moment the host sees it
 *                            every sida_expert_prefetch / forward call returns SIDA_ESTATE until
 *                            sida_pool_reset or sida_set_debug.  The check runs on the stream, so
 *                            it is seen at the latest by the first call after the stream was
 *                            synchronised; sida_debug_mismatch_layer names the layer (-1: none).
 *                            Costs one small launch per layer; the first use allocates one
 *                            pinned host word (not device memory).
 *   SIDA_DEBUG_POISON_SLOTS  a slot that is about to be reloaded is first filled with NaNs (on the
 *                            copy stream, once the last wave that read its old contents is done),
 *                            so that a grouped FFN that ran before its wave's copies were complete
 *                            - a broken wave / event order - shows up as NaN in y instead of as
 *                            stale but plausible numbers (the slot-reuse race between the copy
 *                            and the compute stream is the one race of this design). */
enum { SIDA_DEBUG_CHECK_IDS = 1, SIDA_DEBUG_POISON_SLOTS = 2 };
int sida_set_debug(sida_ctx *ctx, int32_t flags);
int sida_debug_mismatch_layer(const sida_ctx *ctx);

/* Convenience: forwards n consecutive planned layers, keeping the copy stream one wave ahead of
 * the compute across layer boundaries too (the first wave of layer i+1 is copied while the last
 * wave of layer i computes).  plans[i], x_dev[i], ids_dev[i], alpha_dev[i], y_dev[i] belong to
 * the i-th layer of the call; arrays of pointers live in host memory. */
int sida_run_layers(sida_ctx *ctx, int32_t n, const sida_plan *const *plans,
                    const void *const *x_dev, const int32_t *const *ids_dev,
                    const float *const *alpha_dev, void *const *y_dev, void *workspace_dev,
                    size_t workspace_bytes, void *compute_stream, void *copy_stream);

/* ---- single stages (the pieces moe_layer_forward is made of; for tests and profiling) ------- */

/* Counting sort + permute-gather only: fills counts, offsets, perm, inv and x_perm of the
 * workspace for ids_dev / x_dev.  E and d_model come from the context. */
int sida_dispatch(sida_ctx *ctx, const void *x_dev, const int32_t *ids_dev, int32_t T,
                  void *workspace_dev, size_t workspace_bytes, void *stream);
/* Grouped FFN of one local wave of `plan`: reads x_perm and offsets from the workspace (as left
 * by sida_dispatch on the same ids), the experts from their pool slots; writes h and y_perm rows
 * of the wave's experts.  No stream waits, no bookkeeping: the caller guarantees residency. */
int sida_grouped_ffn(sida_ctx *ctx, const sida_plan *plan, int32_t wave, void *workspace_dev,
                     size_t workspace_bytes, void *stream);
/* Gate-weighted scatter-combine only: y[t,:] = alpha[t] * y_perm[inv[t],:]. */
int sida_combine(sida_ctx *ctx, const float *alpha_dev, int32_t T, void *y_dev,
                 void *workspace_dev, size_t workspace_bytes, void *stream);

/* ---- the hash function of the hash-building thread (Section 3.4.2) ----------------------------
 * Predicts the hash table of a batch from the token embeddings alone: for every token and MoE
 * layer the top_k experts and their scaling factors.  Network: a fully connected layer that
 * compresses the embedding to C values, a 2-layer LSTM of width C over the sequence, attention of
 * the LSTM outputs over themselves (dot-product scores) with SparseMax weights, a residual
 * connection adding the token's compressed embedding, and one linear head of E logits per MoE
 * layer; alpha is the SoftMax probability of the expert within its head, the top_k largest are
 * kept (ties to the lower expert id).  All arithmetic in fp32.  No context is needed.
 * params_dev: device fp32, sida_hash_param_count() values packed in this order:
 *   w_in [C, d_model], b_in [C],
 *   LSTM layer 1: w_ih [4C, C], w_hh [4C, C], b_ih [4C], b_hh [4C]   (gate rows: input, forget, cell, output),
 *   LSTM layer 2: the same four,
 *   w_out [L*E, C], b_out [L*E]                                       (head l = rows l*E .. l*E+E-1).
 * x_dev: device bf16 [n_seq * seq_len, d_model], sequences one after the other (attention and the
 * LSTM never cross a sequence boundary).  Outputs, device: ids_dev int32 and alpha_dev fp32, both
 * [L, n_seq * seq_len, top_k] - layer l's slice is exactly the ids / alpha array that
 * sida_moe_plan (after a copy to the host) and sida_moe_layer_forward take (with sida_set_top_k).
 * workspace_dev: device, 256-byte aligned, >= sida_hash_workspace_bytes(n_seq * seq_len).
 * Limits: C is 64 or 128; d_model a multiple of 8, 8 .. 8192; E <= SIDA_MAX_E; L*E <= 8192;
 * top_k <= min(E, SIDA_MAX_TOP_K);
 * seq_len <= max_seq_len <= 4096.  Asynchronous on `stream`. */
typedef struct sida_hash_config {
    int32_t d_model;      /* embedding width                       */
    int32_t C;            /* compressed width = LSTM hidden width  */
    int32_t L, E;         /* MoE layers, experts per layer         */
    int32_t top_k;        /* experts predicted per token and layer */
    int32_t max_seq_len;  /* longest sequence                      */
} sida_hash_config;
size_t sida_hash_param_count(const sida_hash_config *cfg);                       /* 0 on a bad config */
size_t sida_hash_workspace_bytes(const sida_hash_config *cfg, int32_t n_tokens); /* 0 on a bad config */
int sida_hash_forward(const sida_hash_config *cfg, const float *params_dev, const void *x_dev, int32_t n_seq,
                      int32_t seq_len, int32_t *ids_dev, float *alpha_dev, void *workspace_dev,
                      size_t workspace_bytes, void *stream);

/* sida_hash_forward for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels,
 * same results; the intermediates (8*C floats per token) live in a statically allocated device
 * array of SIDA_HASH_STATIC_SCRATCH_BYTES that every GPU the library runs on holds until the
 * process ends.  Calls neither hipMalloc / hipFree nor any other allocating routine; the first
 * call on a device looks the array's address up.  n_seq * seq_len tokens whose intermediates do not
 * fit (more than 4095 tokens at C = 128, 8191 at C = 64) -> SIDA_ENOSPC, nothing enqueued.
 * All calls on one GPU share that GPU's array (it keeps the last call's contents, and nothing in
 * it needs clearing): calls that overlap in time on one GPU - on different streams or from
 * different threads - race; order them on one stream or with events. */
#define SIDA_HASH_STATIC_SCRATCH_BYTES (16u << 20)
int sida_hash_forward_static(const sida_hash_config *cfg, const float *params_dev, const void *x_dev, int32_t n_seq,
                             int32_t seq_len, int32_t *ids_dev, float *alpha_dev, void *stream);

/* Inspection: the order in which a grouped-GEMM launch walks its output tiles.  For a launch over
 * m_tiles token tiles (the first m_tall of them belonging to experts with more than one tile) and
 * n_tiles_n weight-row tiles, fills token_tile[t], weight_tile[t] for t = 0 .. m_tiles*n_tiles_n-1
 * (host arrays); output tile t runs on XCD t % 8.  long_rows != 0: the order of a GEMM whose weight
 * rows are longer than the matrix is tall (an expert's second GEMM).  Host only, no GPU: the device
 * code uses the same function, so tests can check that the order visits every tile exactly once. */
int sida_tile_order(int32_t m_tiles, int32_t m_tall, int32_t n_tiles_n, int32_t long_rows, int32_t *token_tile,
                    int32_t *weight_tile);

/* ---- kernel timing (for the benchmark's roofline figures) ----------------------------------- */

enum { SIDA_K_SORT = 0, SIDA_K_GATHER = 1, SIDA_K_GEMM1 = 2, SIDA_K_GEMM2 = 3, SIDA_K_COMBINE = 4,
       SIDA_K_COPY = 5, SIDA_K_COUNT = 6 };
/* When enabled, every launch (and every wave's batch of copies) is bracketed by timing events on
 * the stream it is enqueued on.  Costs two event records per launch.  Off by default. */
int sida_profile_enable(sida_ctx *ctx, int32_t on);
/* Synchronises the recorded events, adds their durations to the per-class totals and returns the
 * totals since the last reset: ms[SIDA_K_COUNT], launches[SIDA_K_COUNT].  The caller must have
 * synchronised the streams. */
int sida_profile_read(sida_ctx *ctx, double *ms, int64_t *launches, int32_t reset);

#ifdef __cplusplus
}
#endif
#endif /* SIDA_MOE_H */
