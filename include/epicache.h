/*
 * epicache.h - C ABI of the MI355X (gfx950) eviction-step library.
 *
 * One eviction step of EpiCache's block-wise prefill: after a block of M_block
 * tokens has been appended to a cache of at most M entries, the patched-prompt
 * queries of each episode score every context token by the attention it
 * receives, each KV head keeps its top M tokens and the K/V cache is compacted
 * back to M rows (paper Sec. 2.2, Sec. 2.3 Eq. 1, Sec. 3.1 Stage 2, Alg. 1
 * phase A3, App. A.3).  All episodes (and, if the caller folds them into the
 * batch axis, all layers) are processed by one call.
 *
 * Conventions that hold for every entry point
 *   - `params`, `bytes_out`, `keep_capacity_out`, `n_chunks_out` and the arrays
 *     of epicache_layer_budgets are HOST pointers.  Every other pointer is a
 *     DEVICE pointer, 16-byte aligned, owned by the caller.  The library never
 *     allocates, frees or retains device memory and keeps no state between
 *     calls (epicache_evict_step_static and epicache_evict_step_overlapped
 *     document the two exceptions), so it may be called from several host
 *     threads and its calls may be captured into a HIP graph.
 *   - A call validates its arguments on the host, enqueues its kernels on
 *     `hip_stream` (a hipStream_t; NULL = the default stream) and returns
 *     without synchronising.  The return value is an epicache_status; it
 *     covers validation and launch errors only.  On a validation error nothing
 *     has been enqueued.
 *   - Layouts are row-major with the innermost head_dim axis contiguous:
 *       Q      [n_batch, n_q_heads,  patch_len, head_dim]   (strides q_stride_*)
 *       K, V   [n_batch, n_kv_heads, capacity,  head_dim]   (strides kv_stride_*)
 *       scores [n_batch, n_kv_heads, N]            float32, dense
 *       keep   [n_batch, n_kv_heads, n_keep]       int32,   dense
 *     with N = n_cached + n_block context rows and n_keep = min(budget, N).
 *     Strides are in elements and must be multiples of 8; K and V share strides.
 *     Query head hq belongs to KV head hq / (n_q_heads / n_kv_heads).
 *   - Supported: dtype f32 or bf16; head_dim a multiple of 8, 8..256;
 *     N <= 2^24; patch_len * (n_q_heads / n_kv_heads) <= 16384; n_batch * n_kv_heads <= 65535;
 *     token strides <= 2^20 elements.
 *     Anything else returns EPICACHE_ERR_UNSUPPORTED.
 *   - Calls that use the same workspace or the same K/V buffers must be ordered
 *     by the caller (same stream or events).
 *   - One side effect outside the buffers: a bf16 scoring call with more than 8128
 *     scoring rows per KV head (patch_len * n_q_heads / n_kv_heads) needs more than
 *     the default 64 KB of dynamic LDS for one of its kernels and raises that
 *     kernel's limit with hipFuncSetAttribute before the launch (process-wide for
 *     that kernel on the current device, idempotent, not a stream operation).
 */
#ifndef EPICACHE_H
#define EPICACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EPICACHE_API __attribute__((visibility("default")))

typedef enum {
  EPICACHE_OK = 0,
  EPICACHE_ERR_INVALID_ARG = 1,        /* null pointer, non-positive size, bad enum, bad stride */
  EPICACHE_ERR_UNSUPPORTED = 2,        /* valid request outside the supported envelope         */
  EPICACHE_ERR_WORKSPACE_TOO_SMALL = 3,
  EPICACHE_ERR_DEVICE = 4              /* a HIP call failed; hipGetLastError has the detail     */
} epicache_status;

typedef enum { EPICACHE_DTYPE_F32 = 0, EPICACHE_DTYPE_BF16 = 1 } epicache_dtype;

typedef enum {
  EPICACHE_REDUCE_MAX = 0, /* Eq. 1: s_i = max over the scoring queries of Attn(x_t -> x_i) */
  EPICACHE_REDUCE_SUM = 1  /* s_i = sum over the scoring queries (attention mass)           */
} epicache_reduce;

typedef struct epicache_params {
  uint32_t struct_size;   /* sizeof(epicache_params), checked                                 */
  int32_t n_batch;        /* E episodes, or L*E when layers are folded in                     */
  int32_t n_q_heads;      /* Hq, a multiple of n_kv_heads                                     */
  int32_t n_kv_heads;     /* H of the paper                                                   */
  int32_t head_dim;       /* d                                                                */
  int32_t n_cached;       /* rows [0, n_cached): cache kept by the previous step, >= 0        */
  int32_t n_block;        /* rows [n_cached, n_cached+n_block): the new block, >= 0; N >= 1   */
  int32_t budget;         /* M >= 1 (Sec. 2.1)                                                */
  int32_t patch_len;      /* p >= 1 scoring queries per query head (Sec. 2.3)                 */
  int32_t dtype;          /* epicache_dtype of Q, K, V                                        */
  int32_t reduce;         /* epicache_reduce over the G*p rows that vote for one KV head      */
  float softmax_scale;    /* logit scale; 0 selects 1/sqrt(head_dim); at most 1e6             */
  int32_t causal_patch;   /* 0: softmax over the N context keys only.  1: rows [N, N+patch_len) of */
                          /* K[b,h] hold the patch's own keys and patch token t also attends to    */
                          /* patch keys 0..t, as in the model's forward pass (Sec. 2.3); only the  */
                          /* N context rows are scored.  Capacity must then cover N + patch_len.   */
  int32_t reserved;       /* must be 0                                                        */
  int64_t q_stride_b, q_stride_h, q_stride_t;    /* Q strides: batch, head, token             */
  int64_t kv_stride_b, kv_stride_h, kv_stride_t; /* K/V strides; capacity = rows per head     */
} epicache_params;

/* Bytes of device workspace that any of the calls below needs for `params`
 * (the maximum over them, reached by epicache_evict_step with both optional
 * outputs NULL).  Pure host computation. */
EPICACHE_API int epicache_workspace_size(const epicache_params* params, size_t* bytes_out);

/* Sec. 2.3, Eq. 1.  For every batch item b, KV head h and context row i < N:
 * softmax over the N context keys of scale * q.k for each of the G*p query
 * rows of the group, reduced over those rows with `reduce`.
 * In: q, k (read only).  Out: scores [n_batch, n_kv_heads, N] float32.
 * Arithmetic: products and sums in fp32, exponentials in fp32. */
EPICACHE_API int epicache_score(const epicache_params* params, const void* q, const void* k,
                   float* scores, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Sec. 2.3, Eq. 1 with every scoring query's softmax normaliser supplied by the caller: the same
 * scores as epicache_score, computed in a single pass over K.  row_lse [n_batch, n_q_heads,
 * patch_len] float32, dense, read only: natural logarithm of the sum of exp(scale * q.k) over all
 * keys that query attended to, as a fused attention kernel returns it for the patched prompt's
 * forward pass.  If that sum runs over more keys than the N context rows (the patch's own causal
 * keys), the scores are the attention weights under that larger denominator.  Needs the same
 * workspace as epicache_score.  causal_patch must be 0: the supplied normaliser already fixes the
 * denominator. */
EPICACHE_API int epicache_score_lse(const epicache_params* params, const void* q, const void* k,
                   const float* row_lse, float* scores, void* workspace, size_t workspace_bytes,
                   void* hip_stream);

/* Sec. 3.1 Stage 2 / Alg. 1 phase A3 (retention of the M best-scoring tokens).  For every
 * (b, h): the n_keep = min(budget, N) rows with the largest score, written in
 * ascending row order.  Equal scores: the lower row index wins.  Scores are
 * ordered as IEEE-754 totals (-0 < +0, NaN with the sign bit clear above +inf).
 * In: scores [n_batch, n_kv_heads, N].  Out: keep_idx [n_batch, n_kv_heads, n_keep]. */
EPICACHE_API int epicache_topk(const epicache_params* params, const float* scores, int32_t* keep_idx,
                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* Sec. 2.2 / App. A.3 (the cache shrinks back to M entries).  In place, for every
 * (b, h) and j < n_keep:  K[b,h,j,:] = K[b,h,keep_idx[b,h,j],:], same for V.
 * keep_idx must be strictly ascending within [0, N) (as epicache_topk writes
 * it); the order is not checked on the device, and a destination row whose
 * index lies outside [0, N) is left as it is (no access leaves the N rows).
 * Rows >= n_keep are left as they are.  Pure copy, bit exact. */
EPICACHE_API int epicache_compact(const epicache_params* params, const int32_t* keep_idx, void* k, void* v,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/* Alg. 1 phase A3, one block: score -> topk -> compact on one stream, no host
 * synchronisation in between.  scores_opt / keep_idx_opt may be NULL (then the
 * intermediates live in the workspace).  If N <= budget nothing is evicted:
 * keep_idx_opt, if given, is 0..N-1, scores_opt, if given, is still computed,
 * K and V are untouched. */
EPICACHE_API int epicache_evict_step(const epicache_params* params, const void* q, void* k, void* v,
                        float* scores_opt, int32_t* keep_idx_opt, void* workspace,
                        size_t workspace_bytes, void* hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc) and have no workspace at hand: epicache_evict_step with the workspace
 * taken from an array of EPICACHE_STATIC_SCRATCH_BYTES that the library's code object holds in the memory of
 * every GPU it is loaded on, from load until the process ends.  Arguments, results and status codes as
 * epicache_evict_step; the call allocates and frees nothing.  A request whose workspace (what
 * epicache_workspace_size reports, less the parts covered by scores_opt / keep_idx_opt when given) exceeds
 * the array returns EPICACHE_ERR_WORKSPACE_TOO_SMALL and enqueues nothing.  The first call on a device looks
 * up the array's address on that device (the device current at the call must be the one hip_stream belongs
 * to) and keeps it; that table is the only state the library holds.  All calls on one GPU share the one
 * array, which keeps whatever the last call left in it (nothing in it needs to start at zero: every part is
 * written before it is read within a call), so calls that overlap on one GPU, on different streams or from
 * different threads, race: order them on one stream or with events. */
#define EPICACHE_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
EPICACHE_API int epicache_evict_step_static(const epicache_params* params, const void* q, void* k, void* v,
                        float* scores_opt, int32_t* keep_idx_opt, void* hip_stream);

/* Alg. 1 phase A3, one block, as a two-stream pipeline.  The batch is cut into chunks of whole batch items
 * (every (batch item, KV head) of the step is independent, Sec. 3.1 Stage 2); the scoring of chunk c + 1 runs
 * on `hip_stream` while the selection and the in-place compaction of chunk c run on `hip_stream_aux`, so the
 * memory-bound copy proceeds beside the arithmetic-bound scoring instead of after it.  Results as
 * epicache_evict_step, except that the scores may differ from that call's in the last bits (the key splits of
 * the first scoring pass follow the size of the launch, and with them the order of a row's sum).
 *   row_lse_opt      NULL, or the softmax normaliser of every scoring row as epicache_score_lse takes it
 *                    ([n_batch, n_q_heads, patch_len] float32, dense): the scoring is then one pass over K
 *                    (epicache_evict_step_lse over chunks); causal_patch must be 0.
 *   n_chunks         0 = chosen by the library (1, i.e. the plain step, where overlapping does not pay:
 *                    fewer than 256 scoring rows, no MFMA path, or nothing to evict); otherwise 1..64, and
 *                    never more than n_batch.  epicache_overlapped_workspace_size reports the number used
 *                    (with_row_lse: nonzero if row_lse_opt will be given; the library's choice depends on it).
 *   workspace        at least the size epicache_overlapped_workspace_size reports for the same params and
 *                    n_chunks (every chunk has its own slice; scores_opt / keep_idx_opt do not shrink it).
 *   hip_stream_aux   a second stream of the same device, default priority.  Equal to hip_stream: the chunks
 *                    run one after the other on that stream.  HIP multiplexes streams onto a few hardware queues
 *                    (GPU_MAX_HW_QUEUES, 4 by default): in a process with many streams make sure the two do not
 *                    share one, or the step runs serially with the cost of its extra launches on top.
 * Ordering seen by the caller: everything is ordered after the work already enqueued on `hip_stream`, and
 * `hip_stream` waits for the last compaction before the call's successors run, so the call behaves like a
 * single-stream call; `hip_stream_aux` must carry no other work that touches K, V, the workspace, scores_opt
 * or keep_idx_opt.
 * State: the events that order the two streams come from a pool the library creates on the first such call
 * on a device and keeps until the process ends (host-side objects; no device memory).  The device current at
 * the call must be the one both streams belong to.  The call may be captured into a HIP graph from `hip_stream`:
 * `hip_stream_aux` joins the capture through events that live for the call only (the pool is not used then)
 * and leaves it at the join. */
EPICACHE_API int epicache_overlapped_workspace_size(const epicache_params* params, int32_t n_chunks,
                        int32_t with_row_lse, size_t* bytes_out, int32_t* n_chunks_out);
EPICACHE_API int epicache_evict_step_overlapped(const epicache_params* params, const void* q, void* k, void* v,
                        const float* row_lse_opt, float* scores_opt, int32_t* keep_idx_opt, int32_t n_chunks,
                        void* workspace, size_t workspace_bytes, void* hip_stream, void* hip_stream_aux);

/* epicache_evict_step with the scoring done by epicache_score_lse: for callers whose prefill
 * attention kernel already returned each patch row's log-sum-exp (row_lse as documented there).
 * Everything else as epicache_evict_step. */
EPICACHE_API int epicache_evict_step_lse(const epicache_params* params, const void* q, void* k, void* v,
                        const float* row_lse, float* scores_opt, int32_t* keep_idx_opt, void* workspace,
                        size_t workspace_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * Ragged batches: every (batch item, KV head) has its own number of context rows and every batch
 * item its own budget, both read from DEVICE memory, so a sequence of steps needs no host
 * round trip.  Two uses: layers with different budgets (Sec. 3.2, Eq. 6) folded into one launch,
 * and head-wise non-uniform retention (App. A.2, last paragraph: every method in the paper's
 * experiments selects tokens head-wise non-uniformly in the manner of Ada-KV), after which the
 * heads of one layer hold different numbers of rows.
 *
 * In these calls params->n_cached + params->n_block = N_max bounds every context length (it sizes
 * the strides of `scores`, the launch grids and the capacity check) and params->budget bounds
 * every per-item budget.
 *   n_ctx   [n_batch, n_kv_heads] int32: context rows of (b, h); values are clamped to 0..N_max
 *           (with causal_patch the patch keys of (b, h) follow its own context: rows n_ctx .. n_ctx+p-1)
 *   budgets [n_batch] int32: M_b, clamped to 1..params->budget; NULL = params->budget everywhere
 *   scores  [n_batch, n_kv_heads, N_max] float32: entries at or beyond n_ctx[b,h] are not written
 *   keep    [n_batch, n_kv_heads, keep_capacity] int32: the first n_kept[b,h] entries are valid
 *   n_kept  [n_batch, n_kv_heads] int32 (out): rows (b, h) holds after the step
 * keep_capacity = min(budget, N_max) for EPICACHE_SELECT_PER_HEAD and
 * min(n_kv_heads * budget, N_max) for EPICACHE_SELECT_POOLED.
 * Pooled selection additionally needs n_kv_heads <= 1024 and n_kv_heads * N_max < 2^31. */
typedef enum {
  EPICACHE_SELECT_PER_HEAD = 0, /* each (b, h) keeps its min(M_b, n_ctx) best rows (Sec. 3.1 Stage 2)   */
  EPICACHE_SELECT_POOLED = 1    /* the heads of item b share one pool: its min(Hkv * M_b, sum of n_ctx)  */
                                /* best entries are kept; ties: lower head, then lower row (App. A.2)    */
} epicache_select;

/* Workspace bytes for the ragged calls below and the row pitch of `keep`.  Pure host computation. */
EPICACHE_API int epicache_ragged_workspace_size(const epicache_params* params, int32_t select,
                                                size_t* bytes_out, int32_t* keep_capacity_out);

/* Eq. 1 as epicache_score, over the first n_ctx[b,h] rows of K[b,h].  Rows with n_ctx = 0 get no
 * scores.  row_lse_opt: NULL, or the caller's row normalisers as in epicache_score_lse (single pass
 * over K; causal_patch must then be 0). */
EPICACHE_API int epicache_score_ragged(const epicache_params* params, const void* q, const void* k,
                                       const int32_t* n_ctx, const float* row_lse_opt, float* scores,
                                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* Retention on given scores.  Writes keep (ascending within each head) and n_kept.  Score order and
 * per-head tie rule as epicache_topk. */
EPICACHE_API int epicache_select_ragged(const epicache_params* params, int32_t select, const float* scores,
                                        const int32_t* n_ctx, const int32_t* budgets, int32_t* keep_idx,
                                        int32_t* n_kept, void* workspace, size_t workspace_bytes,
                                        void* hip_stream);

/* In-place compaction as epicache_compact with n_kept[b,h] rows per head; `select` only fixes the
 * row pitch of keep_idx. */
EPICACHE_API int epicache_compact_ragged(const epicache_params* params, int32_t select,
                                         const int32_t* keep_idx, const int32_t* n_kept, void* k, void* v,
                                         void* workspace, size_t workspace_bytes, void* hip_stream);

/* score_ragged -> select_ragged -> compact_ragged on one stream.  n_kept is required: it is the
 * n_cached of each head for the next step (n_ctx_next = n_kept + next block).  row_lse_opt as in
 * epicache_score_ragged.  scores_opt and keep_idx_opt may be NULL. */
EPICACHE_API int epicache_evict_step_ragged(const epicache_params* params, int32_t select, const void* q,
                                            void* k, void* v, const int32_t* n_ctx, const int32_t* budgets,
                                            const float* row_lse_opt, int32_t* n_kept, float* scores_opt,
                                            int32_t* keep_idx_opt, void* workspace, size_t workspace_bytes,
                                            void* hip_stream);

/* epicache_evict_step_ragged as a two-stream pipeline over chunks of whole batch items, exactly as
 * epicache_evict_step_overlapped does it for the uniform step (scoring of chunk c + 1 on `hip_stream` beside the
 * selection and compaction of chunk c on `hip_stream_aux`; same ordering, state, capture and n_chunks rules, with
 * N_max and params->budget in the place of N and M).  Every array is used in slices of whole batch items.  The
 * workspace size, the keep capacity (as epicache_ragged_workspace_size reports it) and the number of chunks used come
 * from epicache_ragged_overlapped_workspace_size. */
EPICACHE_API int epicache_ragged_overlapped_workspace_size(const epicache_params* params, int32_t select,
                                            int32_t n_chunks, int32_t with_row_lse, size_t* bytes_out,
                                            int32_t* keep_capacity_out, int32_t* n_chunks_out);
EPICACHE_API int epicache_evict_step_ragged_overlapped(const epicache_params* params, int32_t select, const void* q,
                                            void* k, void* v, const int32_t* n_ctx, const int32_t* budgets,
                                            const float* row_lse_opt, int32_t* n_kept, float* scores_opt,
                                            int32_t* keep_idx_opt, int32_t n_chunks, void* workspace,
                                            size_t workspace_bytes, void* hip_stream, void* hip_stream_aux);

/* Sec. 2.3: the patched prompt's own pass through the attention layer.  For every patch query t of every
 * query head: out[b,hq,t,:] = sum_i softmax_i(scale * q.k_i) V[b,h,i,:] and lse_out[b,hq,t] = natural log of
 * sum_i exp(scale * q.k_i), over the N context rows and, with causal_patch = 1, the patch rows 0..t that
 * follow them (rows N .. N+patch_len-1 of K and V).  lse_out is exactly the row_lse that epicache_score_lse /
 * epicache_evict_step_lse take (call those with causal_patch = 0), so this call plus
 * epicache_evict_step_lse is the patch's attention, Eq. 1 scoring, selection and compaction with K read twice.
 * In: q, k, v (read only; V has the strides of K).  Out: out [n_batch, n_q_heads, patch_len, head_dim]
 * in the dtype of the inputs, dense; lse_out [n_batch, n_q_heads, patch_len] float32, dense.
 * bf16 with head_dim 128 runs on the matrix cores (weights rounded to bf16 before the product with V, fp32
 * accumulation); other dtypes / head dims take a plain fp32 kernel.  No workspace. */
EPICACHE_API int epicache_patch_attention(const epicache_params* params, const void* q, const void* k,
                                          const void* v, void* out, float* lse_out, void* hip_stream);

/* Sec. 2.3 on caches whose heads hold different numbers of tokens (head-wise non-uniform retention,
 * App. A.2): epicache_patch_attention with the context length of head (b, h) read from
 * n_ctx[b * n_kv_heads + h] (device memory, int32, clamped to [0, n_cached + n_block]); with
 * causal_patch = 1 the patch rows of that head follow its own context (rows n_ctx .. n_ctx + patch_len - 1).
 * A query without a single key (empty context, causal_patch = 0) gets out = 0 and lse_out = -inf.
 * lse_out is what epicache_score_ragged / epicache_evict_step_ragged take as row_lse_opt. */
EPICACHE_API int epicache_patch_attention_ragged(const epicache_params* params, const void* q, const void* k,
                                                 const void* v, const int32_t* n_ctx, void* out, float* lse_out,
                                                 void* hip_stream);

/* Alg. 1 phase A3 with the patch's forward pass folded in: epicache_patch_attention (out as documented there;
 * the normalisers stay in the workspace) followed by the single-pass scoring on those normalisers, the
 * top-M selection and the in-place compaction, on one stream.  With causal_patch = 1 the denominators are the
 * model's own (context keys and the patch's causal keys, rows N .. N+patch_len-1 of K and V, which are never
 * scored or kept); with 0 they are those of epicache_evict_step.  K is read twice, V once before it is
 * compacted.  scores_opt / keep_idx_opt and the N <= budget case as in epicache_evict_step. */
EPICACHE_API int epicache_evict_step_attn(const epicache_params* params, const void* q, void* k, void* v,
                                          void* out, float* scores_opt, int32_t* keep_idx_opt, void* workspace,
                                          size_t workspace_bytes, void* hip_stream);

/* App. A.2 ("SnapKV" inside block prefill): Eq. 1 with the block's own last w = patch_len tokens, the
 * observation window, as the patched prompt.  The window rows are the last w of the N = n_cached + n_block
 * context rows of K and V; q_window [n_batch, n_q_heads, w, head_dim] holds their query states (strides
 * q_stride_*).  Window token t sits at row N - w + t and attends to rows 0 .. N - w + t, itself included, as
 * in the model's forward pass; only the N - w rows before the window are scored, the window rows are always
 * retained, and the budget - w best earlier rows are kept next to them, in row order (the paper says no more
 * than that the window is the patched prompt; keeping the window is SnapKV's own design).
 * Requires budget > w whenever N > budget (else EPICACHE_ERR_INVALID_ARG) and params->causal_patch = 0 (the
 * call applies the window's mask itself).
 * Out: scores_opt [n_batch, n_kv_heads, N - w] (nothing if N <= w), keep_idx_opt [n_batch, n_kv_heads,
 * min(budget, N)]; both may be NULL.  K, V compacted in place.  If N <= budget nothing is evicted. */
EPICACHE_API int epicache_snapkv_workspace_size(const epicache_params* params, size_t* bytes_out);
EPICACHE_API int epicache_evict_step_snapkv(const epicache_params* params, const void* q_window, void* k, void* v,
                                            float* scores_opt, int32_t* keep_idx_opt, void* workspace,
                                            size_t workspace_bytes, void* hip_stream);

/* App. A.2 ("KVzip" inside block prefill): Eq. 1 with a repetition instruction followed by the whole block as
 * the patched prompt, i.e. a patch of thousands of tokens per query head.  Same scores as epicache_score, but
 * patch_len may be anything up to 2^20 (n_q_heads / n_kv_heads <= 4096): every scoring row is normalised on
 * its own, so the patch tokens are scored 4096 / (n_q_heads / n_kv_heads) at a time and the chunks' score
 * vectors are combined with `reduce`.  causal_patch must be 0.  Results, optional outputs and the N <= budget
 * case of epicache_evict_step_kvzip as epicache_evict_step. */
EPICACHE_API int epicache_kvzip_workspace_size(const epicache_params* params, size_t* bytes_out);
EPICACHE_API int epicache_score_kvzip(const epicache_params* params, const void* q, const void* k, float* scores,
                                      void* workspace, size_t workspace_bytes, void* hip_stream);
EPICACHE_API int epicache_evict_step_kvzip(const epicache_params* params, const void* q, void* k, void* v,
                                           float* scores_opt, int32_t* keep_idx_opt, void* workspace,
                                           size_t workspace_bytes, void* hip_stream);

/* App. A.2 ("KeyDiff"): the attention-free baseline scorer, for the same epicache_topk /
 * epicache_compact (or *_ragged) back end.  Per (b, h): anchor = mean of the key states of the
 * context rows; scores[b,h,i] = -cos(K[b,h,i,:], anchor), so the keys that point away from the bulk
 * score highest.  A zero key or a zero anchor gives 0.  Sums and products in fp32.
 * n_ctx_opt: NULL, or per-(b,h) lengths [n_batch, n_kv_heads] as in the ragged calls (then
 * n_cached + n_block is their upper bound and the pitch of a score row).  The query fields of
 * params are not used but must still be valid (for instance n_q_heads = n_kv_heads, patch_len = 1). */
EPICACHE_API int epicache_score_keydiff(const epicache_params* params, const void* k, const int32_t* n_ctx_opt,
                                        float* scores, void* workspace, size_t workspace_bytes,
                                        void* hip_stream);

/* Sec. 3.1 Stage 1, Eq. 3: for every cluster e of segment embeddings, its centroid (mean of the member
 * embeddings) and its centroid-closest member (largest cosine to the centroid; equal cosines: the
 * lower segment index), the segment that serves as the episode's patched prompt.  The encoder and the
 * clustering are the caller's: embeddings [n_segments, dim] fp32 and assignment [n_segments] int32 in
 * 0..n_episodes-1 are inputs (values outside that range belong to no cluster).  Out: centroids_out
 * [n_episodes, dim] fp32 and medoid_out [n_episodes] int32; an empty cluster gets a zero centroid and
 * medoid -1.  All DEVICE pointers, dense.  dim <= 8192. */
EPICACHE_API int epicache_episode_medoids(const float* embeddings, const int32_t* assignment,
                                          int32_t n_segments, int32_t n_episodes, int32_t dim,
                                          float* centroids_out, int32_t* medoid_out, void* hip_stream);

/* Sec. 3.1 Stage 3a: episode_out[i] = argmax over e of cos(queries[i], centroids[e]) (equal cosines: the
 * lower e); Stage 3b: -1 instead when that cosine is below tau (the query opens a new episode; pass
 * -INFINITY to always match).  The cosine with a zero vector is 0.  cosine_out_opt, if not NULL,
 * receives the best cosine.  queries [n_queries, dim], centroids [n_episodes, dim] fp32, dense, DEVICE. */
EPICACHE_API int epicache_match_queries(const float* queries, const float* centroids, int32_t n_queries,
                                        int32_t n_episodes, int32_t dim, float tau, int32_t* episode_out,
                                        float* cosine_out_opt, void* hip_stream);

/* Sec. 3.2, Eq. 6 / Alg. 1 phase A2: split the global budget n_layers * budget over the layers in
 * proportion to sensitivity[l]^alpha (sensitivity[l] = 1 - sigma_l >= 0, alpha >= 0 the sharpness).
 * The paper's allocation is real-valued; here it is rounded by largest remainder (ties to the lower
 * layer) so that the integers sum to n_layers * budget exactly, and no layer is left below one row
 * (a row is taken from the currently largest layer for each layer that would get none).  All-zero
 * sensitivities give the uniform split.  HOST pointers, pure host computation; budgets_out[l] is
 * the `budget` to pass to the calls above for layer l. */
EPICACHE_API int epicache_layer_budgets(const double* sensitivity, int32_t n_layers, double alpha,
                                        int32_t budget, int32_t* budgets_out);

/* Static, NUL-terminated description of an epicache_status value. */
EPICACHE_API const char* epicache_status_string(int status);

/* Library version, "major.minor.patch". */
EPICACHE_API const char* epicache_version(void);

#ifdef __cplusplus
}
#endif
#endif /* EPICACHE_H */
