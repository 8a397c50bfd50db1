/*
 * fastcache.h - C ABI of the batched KV-cache compression stage for MI355X.
 *
 * The stage is the "batch compression" step of FastCache's serving loop
 * (Algorithm 1: kv <- P.Store(M.Prefill(batch)); kv_c <- C(kv, lambda);
 * decode; P.Release(kv_c)) together with the KV-cache memory pool it works on
 * ("KV-cache Memory Pool" paragraph of the Dynamic Resource Management
 * section: the pool reclaims the pre-compression "zombie" caches right after
 * compression and manages the compressed ones centrally).  Stage hand-off is
 * by block tables, i.e. by reference ("zero-copy mechanism", System
 * Implementation section); the only data movement is the compaction copy.
 *
 * Every function returns FC_OK (0) or a negative error code.  FC_EINVAL and
 * FC_ENOMEM are raised before anything is queued: the pool, its free list and
 * all caller buffers are left unchanged.  FC_EDEVICE (a HIP call failed) is
 * different: if it comes from a launch in the middle of a stage, part of the
 * stage's device work is already queued while the host mirrors (free count,
 * lengths) were not advanced; the pool is then marked unusable, every later
 * call on it returns FC_EDEVICE, and the caller has to destroy it and rebuild
 * its block tables.  The library's scratch buffers (kept lists, saved ids,
 * un-pooled scores, descriptors) grow on demand: a call that needs more than
 * any earlier one waits for the device, frees and reallocates BEFORE it queues
 * anything; calls whose needs were met before are fully asynchronous.
 * "dev" pointers are device (HBM) addresses, "host" pointers are ordinary
 * host memory.  All device work is issued on the hipStream_t passed as
 * `stream` (NULL = the default stream) and is asynchronous with respect to
 * the host unless stated otherwise.  A pool is not thread safe: calls on one
 * pool must be serialised by the caller, and work on different streams must
 * be ordered by the caller.
 */
#ifndef FASTCACHE_H
#define FASTCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fc_pool fc_pool; /* opaque, owned by the library */

enum { FC_OK = 0, FC_EINVAL = -1, FC_ENOMEM = -2, FC_EDEVICE = -3 };
enum { FC_METHOD_NONE = 0, FC_METHOD_SNAPKV = 1, FC_METHOD_KNORM = 2, FC_METHOD_STREAMING = 3 };
enum { FC_DTYPE_F16 = 0 };

#define FC_BLOCK_SIZE 16      /* tokens per pool block (the only supported value) */
#define FC_MAX_WINDOW 64      /* largest observation window */
#define FC_MAX_SEQ_LEN 32768  /* longest request the stage accepts */
#define FC_MAX_POOL_KERNEL 63 /* largest max-pool kernel */

/*
 * Creates a pool over caller-owned device memory (Algorithm 1, "Initialize
 * KVCachePool P").
 *
 * kv_base   dev, caller-owned for the lifetime of the pool, 256-byte aligned,
 *           fp16, laid out as
 *             kv[layer][block][kv: 0=K, 1=V][head][slot 0..15][head_dim]
 *           so that (layer, block, kv, head) is one contiguous chunk of
 *           16*head_dim halves.  The engine writes prefill K/V rows straight
 *           into it; token j of a request lives in block table[j / 16],
 *           slot j % 16, for every layer and head.
 * kv_bytes  size of that memory; must be >= n_layers*n_blocks*2*n_heads*16*
 *           head_dim*2.
 * block_size must be 16, head_dim 64 or 128, dtype FC_DTYPE_F16.
 *
 * The free list is a LIFO stack of block ids held in device memory; a fresh
 * pool holds stack[i] = n_blocks-1-i, top = n_blocks, so that the first
 * block handed out is block 0.  Synchronous.
 */
int fc_pool_create(fc_pool** out, void* kv_base, size_t kv_bytes, int n_blocks,
                   int block_size, int n_layers, int n_heads, int head_dim,
                   int dtype);

/* Releases the library's own device memory (free list, scratch).  Waits for
 * the device first.  kv_base stays the caller's. */
int fc_pool_destroy(fc_pool* pool);

/*
 * P.Store side of the pool: pops n_blocks ids off the free stack,
 * dev_out_ids[i] = stack[top-1-i], then top -= n_blocks.
 * dev_out_ids: dev, int32[n_blocks], caller-owned.
 * FC_ENOMEM if fewer than n_blocks are free, FC_EINVAL if n_blocks < 0.
 */
int fc_pool_alloc(fc_pool* pool, int n_blocks, int32_t* dev_out_ids, void* stream);

/*
 * P.Release: pushes ids in array order, stack[top+i] = dev_ids[i], then
 * top += n_blocks.  dev_ids: dev, int32[n_blocks].  The ids must have come
 * from this pool and be owned by the caller (checked only with
 * fc_set_debug_checks); FC_EINVAL if the push would exceed the pool size.
 */
int fc_pool_free(fc_pool* pool, const int32_t* dev_ids, int n_blocks, void* stream);

/*
 * Ownership checks, a debug mode for the pool's invariant that every block is
 * either on the free stack or owned by exactly one request ("KV-cache Memory
 * Pool" paragraph: the pool is the one authority over allocation and release).
 * With the checks on, the library keeps one word per block on the device
 * (free / handed out) and
 *   - fc_pool_free, and the release of the old blocks inside fc_compress_batch
 *     (all variants) and fc_compress_batch_mlp, first verify every id they are
 *     about to push: inside the pool, currently handed out, named once.  A
 *     double free, a foreign or free id, or a duplicate gives FC_EINVAL and
 *     nothing is changed.  These calls then wait for the device once (the
 *     verdict is read on the host), so they are no longer asynchronous;
 *   - every pop (fc_pool_alloc, the new blocks of a compression, fc_append_batch)
 *     marks its blocks handed out and raises a flag if one of them was not
 *     free; fc_pool_export_state reports the flag as FC_EDEVICE.
 * Switching the checks on takes what is on the free stack as free and every
 * other block as handed out (so does fc_pool_import_state); it waits for the
 * device.  Off by default: block ids are then only clamped into the pool.
 */
int fc_set_debug_checks(fc_pool* pool, int enable);

/* Number of free blocks (exact host-side mirror of top), or a negative error. */
int fc_pool_num_free(const fc_pool* pool);

/*
 * Copies the free stack to host_stack (host, int32[n_blocks]; entries
 * [0, *top) are meaningful) after waiting for all device work.  Synchronous.
 * Also reports, as FC_EDEVICE, a finding of the ownership checks on a pop
 * (a block that came off the free stack was not free).  Such a condition is
 * reported by one call (which copies nothing) and cleared; the next call
 * succeeds unless it has happened again.
 */
int fc_pool_export_state(fc_pool* pool, int32_t* host_stack, int* top);

/* Overwrites the free stack and top from the host (used to rewind metadata
 * between benchmark repetitions).  0 <= top <= n_blocks.  Synchronous. */
int fc_pool_import_state(fc_pool* pool, const int32_t* host_stack, int top);

/* Same from a device copy of the stack (dev, int32[n_blocks]), asynchronously
 * on `stream`, so that a benchmark can rewind without idling the GPU. */
int fc_pool_import_state_dev(fc_pool* pool, const int32_t* dev_stack, int top, void* stream);

/*
 * kv_c <- C(kv, lambda) for a whole batch (Algorithm 1, "Batch compression";
 * Pipeline Optimization section: compression of many requests is issued as
 * one grouped operation instead of one launch sequence per request).
 *
 * For every request r with method != FC_METHOD_NONE, every layer and head:
 *   1. score the L_r cached tokens
 *        FC_METHOD_SNAPKV: queries of the last `window` tokens attend (causal,
 *          logits scale*q.k, row softmax) over the cached keys; per key, sum
 *          over the window queries; max-pool (odd pool_kernel, stride 1, same
 *          length) over the keys before the window; window tokens score +inf;
 *        FC_METHOD_KNORM: score = -||k||_2;
 *        FC_METHOD_STREAMING (StreamingLLM-style baseline of the paper's
 *          evaluation): nothing is read; the first min(n_sink, budget_r)
 *          tokens and the last budget_r - sinks tokens score +inf, the rest 0
 *          (n_sink: fc_set_streaming_sinks, default 4);
 *   2. keep the budget_r best scores (ties to the lower index), in ascending
 *      token order;
 *   3. pop ceil(budget_r/16) new blocks (all requests' new blocks are popped
 *      first, in batch order), copy the kept K and V rows densely into them;
 *   4. push the request's old blocks (batch order, table order) back on the
 *      free stack, rewrite its block-table row (entries past the new count
 *      become -1) and set host_seq_lens[r] = budget_r.
 *
 * dev_block_tables  dev, int32 [n_req][max_blocks_per_req], in/out.
 * host_seq_lens     host, int32 [n_req], in/out (updated before returning).
 * dev_q_window      dev, fp16 [n_req][n_layers][n_heads][window][head_dim],
 *                   16-byte aligned; may be NULL if no request uses SNAPKV.
 * host_method, host_budget  host, int32 [n_req].
 * pool_kernel       odd, 1..FC_MAX_POOL_KERNEL.   scale <= 0 means
 *                   1/sqrt(head_dim).
 * dev_scores_out    dev or NULL: final fp32 scores packed as
 *                   [r][layer][head][L_r] over the compressed requests in
 *                   batch order (request r starts at the sum over earlier
 *                   compressed requests of L*n_layers*n_heads).
 * dev_kept_out      dev or NULL: kept indices, int32, packed the same way
 *                   with budget_r in place of L_r.
 *
 * FC_EINVAL: unknown method; budget < 1 or > L; L > FC_MAX_SEQ_LEN; SNAPKV
 * with window outside 1..FC_MAX_WINDOW, L < window or budget < window;
 * ceil(L/16) > max_blocks_per_req; bad pool_kernel; NULL where a buffer is
 * needed.  FC_ENOMEM: the sum of new blocks exceeds the free blocks (new
 * blocks are taken before old ones are released because the copy reads the
 * old blocks while it writes the new ones).  FC_EDEVICE: a HIP call failed.
 */
int fc_compress_batch(fc_pool* pool, int32_t* dev_block_tables, int max_blocks_per_req,
                      int32_t* host_seq_lens, const void* dev_q_window, int window,
                      const int32_t* host_method, const int32_t* host_budget, int n_req,
                      int pool_kernel, float scale, float* dev_scores_out,
                      int32_t* dev_kept_out, void* stream);

/*
 * fc_compress_batch for callers that cannot allocate device memory while they
 * call it: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same results (the same kernels run), but
 * every scratch buffer of the call (kept lists, saved and new block ids,
 * request descriptors) lies in ONE fixed device array of
 * FC_NOALLOC_SCRATCH_BYTES that the library's code object holds on every GPU
 * it is loaded on until the process ends; the call allocates and frees
 * nothing, on the device or in pinned host memory, and never waits for the
 * device.  Limits (FC_EINVAL beyond them, nothing touched):
 *   - at most FC_NOALLOC_MAX_REQUESTS compressed requests per call;
 *   - every compressed request has at most 8192 tokens and the pool uses the
 *     default scheduling (FC_SCORE_AUTO): nothing may need the library's
 *     un-pooled score scratch;
 *   - sum over requests of budget * n_layers * n_heads <= 15 Mi entries,
 *     unless dev_kept_out is given (then the kept lists go there);
 *   - sum over requests of ceil(L/16) + ceil(budget/16) <= 256 Ki block ids.
 * All calls on one GPU share that GPU's array and it keeps the last call's
 * contents (nothing in it has to start at zero): two such calls that overlap
 * in time on one GPU, on any streams or pools, race.
 */
#define FC_NOALLOC_MAX_REQUESTS 64
#define FC_NOALLOC_SCRATCH_BYTES ((15u << 20) * 4u + (256u << 10) * 4u + (16u << 10))
int fc_compress_batch_noalloc(fc_pool* pool, int32_t* dev_block_tables, int max_blocks_per_req,
                              int32_t* host_seq_lens, const void* dev_q_window, int window,
                              const int32_t* host_method, const int32_t* host_budget, int n_req,
                              int pool_kernel, float scale, float* dev_scores_out,
                              int32_t* dev_kept_out, void* stream);

/*
 * The same stage (Algorithm 1, "Batch compression") for a batch whose SnapKV
 * requests each have their own observation window and max-pool width, as
 * when requests come from models or prompts with different settings.
 *
 * host_window, host_pool_kernel  host, int32 [n_req]; entry r is looked at
 *                   only if host_method[r] == FC_METHOD_SNAPKV (window in
 *                   1..FC_MAX_WINDOW, pool width odd in 1..FC_MAX_POOL_KERNEL).
 * dev_q_window      dev, fp16, 16-byte aligned, packed in batch order over the
 *                   SnapKV requests only: request r contributes
 *                   [n_layers][n_heads][host_window[r]][head_dim].
 * Everything else, including errors, as for fc_compress_batch.
 */
int fc_compress_batch_var(fc_pool* pool, int32_t* dev_block_tables, int max_blocks_per_req,
                          int32_t* host_seq_lens, const void* dev_q_window,
                          const int32_t* host_window, const int32_t* host_method,
                          const int32_t* host_budget, const int32_t* host_pool_kernel, int n_req,
                          float scale, float* dev_scores_out, int32_t* dev_kept_out,
                          void* stream);

/*
 * The pruning stage (Algorithm 1, "Batch compression") when the caller already
 * has the soft-max denominators of the observation-window rows.  The prefill
 * that comes right before the stage in Algorithm 1 (M.Prefill) runs attention
 * for exactly these queries over exactly these keys, and fused attention
 * kernels return, per query row, the natural logarithm of the sum of
 * exp(logit) over the keys the row sees.  With that number the score of key j,
 * sum_i exp(scale * q_i . k_j - lse_i), needs one pass over K instead of two.
 *
 * dev_lse_window    dev, fp32 [n_req][n_layers][n_heads][window], 4-byte
 *                   aligned; entry i of a unit = log(sum over keys j at
 *                   positions <= L - window + i of exp(scale * q_i . k_j)),
 *                   with the same scale as this call.  Read for SNAPKV requests
 *                   only.  The library does not check it: a row whose entry is
 *                   off by t contributes exp(-t) times its soft-max row.
 * Everything else, including errors, as for fc_compress_batch; additionally
 * FC_EINVAL if a SNAPKV request is present and dev_lse_window is NULL.
 */
int fc_compress_batch_lse(fc_pool* pool, int32_t* dev_block_tables, int max_blocks_per_req,
                          int32_t* host_seq_lens, const void* dev_q_window,
                          const float* dev_lse_window, int window, const int32_t* host_method,
                          const int32_t* host_budget, int n_req, int pool_kernel, float scale,
                          float* dev_scores_out, int32_t* dev_kept_out, void* stream);

/*
 * The row log-sum-exp that fc_compress_batch_lse takes, computed from the pool
 * (one pass over K; the first half of what fc_compress_batch does for a SNAPKV
 * request), for callers whose attention kernel does not return it.  Reads the
 * pool, changes nothing: no allocation, tables and lengths untouched.
 *
 * dev_block_tables, max_blocks_per_req, host_seq_lens, dev_q_window, window,
 * scale             as for fc_compress_batch (host_seq_lens is read only).
 * host_method       host, int32 [n_req] or NULL: rows are computed for requests
 *                   with FC_METHOD_SNAPKV (all requests if NULL).
 * dev_lse_out       dev, fp32 [n_req][n_layers][n_heads][window]; rows of the
 *                   other requests are left as they are.
 * FC_EINVAL: window outside 1..FC_MAX_WINDOW, a computed request with L < window,
 * L > FC_MAX_SEQ_LEN or ceil(L/16) > max_blocks_per_req, NULL or misaligned
 * buffers.  Asynchronous on `stream`.
 */
int fc_window_lse(fc_pool* pool, const int32_t* dev_block_tables, int max_blocks_per_req,
                  const int32_t* host_seq_lens, const void* dev_q_window, int window,
                  const int32_t* host_method, int n_req, float scale, float* dev_lse_out,
                  void* stream);

/*
 * The paper's own compressor shape ("Multimodal Compressor" section): the cache
 * is split at the modality boundary, every run of k consecutive tokens of one
 * modality is reshaped into one vector of k*head_dim numbers and mapped to ONE
 * row by that modality's MLP, and the results are concatenated in the
 * original order.  The paper gives neither architecture, activation nor
 * weights; this library takes  y = W2 . act(W1 . x + b1) + b2  (one hidden
 * layer) with caller-supplied weights, shared by all layers, heads and by K
 * and V, and the activation as an argument:
 *   FC_ACT_GELU_ERF   GELU by its definition, v * Phi(v) = v/2 (1 + erf(v/sqrt 2));
 *   FC_ACT_GELU_TANH  its tanh approximation,
 *                     v/2 (1 + tanh(sqrt(2/pi) (v + 0.044715 v^3))).
 * Arithmetic: fp16 rows and weights, fp32 accumulation, the hidden activations
 * are held in fp16, the output is stored in fp16 (the pool's type): a stored
 * value y_c differs from the exact one by at most about
 *   2^-11 |y_c| + sum_u |W2[c][u]| (2^-11 |h_u| + 1e-4).
 * head_dim 64 or 128; hidden 128 or 256; k in 1..8.
 */
enum { FC_ACT_GELU_ERF = 0, FC_ACT_GELU_TANH = 1 };
typedef struct fc_mlp_weights {
  int k;              /* tokens per chunk = compression factor */
  int hidden;         /* hidden width */
  int activation;     /* FC_ACT_* */
  const void* w1[2];  /* dev, fp16 [hidden][k*head_dim] row-major; [0] text, [1] image */
  const float* b1[2]; /* dev, fp32 [hidden] */
  const void* w2[2];  /* dev, fp16 [head_dim][hidden] row-major */
  const float* b2[2]; /* dev, fp32 [head_dim] */
} fc_mlp_weights;

/* Copies the weights into library-owned device memory in the operand order of
 * the kernel (the caller's buffers may be released after the stream has run
 * past this call).  FC_EINVAL for unsupported sizes, an unknown activation or
 * NULL pointers. */
int fc_mlp_set_weights(fc_pool* pool, const fc_mlp_weights* weights, void* stream);

/*
 * Chunk-MLP compression of a whole batch.  Request r (if host_enable is NULL
 * or host_enable[r] != 0) has text tokens [0, img_begin_r), image tokens
 * [img_begin_r, img_end_r) and text tokens [img_end_r, L_r); each of the three
 * segments is cut into ceil(n/k) chunks (the last one zero-padded) and every
 * chunk becomes one row, for every layer and head, K and V alike.  New blocks
 * for ceil(L'_r/16) rows (L'_r = number of chunks) are popped for all
 * requests first, then all old blocks are pushed, exactly as in
 * fc_compress_batch; host_seq_lens[r] becomes L'_r.  Block-table and length
 * arguments as in fc_compress_batch.  FC_EINVAL: weights not set, bad span,
 * table too small; FC_ENOMEM: not enough free blocks.
 */
int fc_compress_batch_mlp(fc_pool* pool, int32_t* dev_block_tables, int max_blocks_per_req,
                          int32_t* host_seq_lens, const int32_t* host_img_begin,
                          const int32_t* host_img_end, const int32_t* host_enable, int n_req,
                          void* stream);

/*
 * Where fc_compress_batch puts the kept rows.
 *   FC_COMPACT_FRESH (default): into freshly popped blocks, as described at
 *     fc_compress_batch (needs sum ceil(budget_r/16) free blocks).
 *   FC_COMPACT_IN_PLACE: into the request's own first ceil(budget_r/16) blocks
 *     (kept row t moves to slot t; rows are moved in ascending chunks so that
 *     no row is overwritten before it has been read).  No block is popped,
 *     FC_ENOMEM cannot occur, the table row keeps its first ceil(budget_r/16)
 *     ids and the remaining ids are pushed on the free stack (batch order,
 *     table order).  For pools that are nearly full.
 */
enum { FC_COMPACT_FRESH = 0, FC_COMPACT_IN_PLACE = 1 };
int fc_set_compaction_mode(fc_pool* pool, int mode);

/* Number of leading "attention sink" tokens that FC_METHOD_STREAMING requests
 * keep (>= 0, default 4). */
int fc_set_streaming_sinks(fc_pool* pool, int n_sink);

/*
 * How fc_compress_batch schedules the scoring.
 *   FC_SCORE_AUTO (default): every (request, layer, head) of at most 8192
 *     tokens is handled by one fused kernel (two-pass score -> select -> gather
 *     inside the workgroup that owns the head; scores stay in LDS); longer
 *     heads go through the separate two-pass score, select and gather kernels.
 *     (See fc_set_score_pruning for what the fused kernel does with the
 *     second pass when the call does not ask for the scores.)
 *   FC_SCORE_TWO_PASS: separate kernels for everything; SnapKV scoring streams
 *     K twice (row statistics, then column sums); any length up to
 *     FC_MAX_SEQ_LEN.
 * Both produce the same scores up to fp32 rounding.  In neither does a
 * workgroup ever wait for another one.
 */
enum { FC_SCORE_AUTO = 0, FC_SCORE_TWO_PASS = 1 };
int fc_set_score_mode(fc_pool* pool, int mode);

/*
 * Pruned second pass of the SnapKV-style score (Algorithm 1, "Batch
 * compression"; the selection only needs exact scores near its threshold).
 * On by default (enable == 0 turns it off): for heads of at least 512 tokens
 * the fused kernel of the default
 * scheduling bounds every column sum during its first pass over K and re-reads
 * only the key rows whose exact score can still decide the selection.  The kept
 * set is the exact top-budget set of the exactly evaluated scores, as on the
 * two-pass path (the two evaluate a column sum in different orders of
 * addition, so between scores that agree to fp32 rounding the choice may
 * differ); the compacted caches and the pool follow from it in the same way.
 * It applies to calls that do not ask for the scores (dev_scores_out == NULL)
 * and do not bring the row log-sum-exps; the separate-kernel modes never
 * prune.  The bounds live in the kernel's local memory: no device memory
 * beyond that of the two-pass path is used.
 */
int fc_set_score_pruning(fc_pool* pool, int enable);

/*
 * Per-kernel timing for benchmarks.  With profiling enabled every kernel
 * launched by fc_compress_batch is bracketed by HIP events on the call's
 * stream; the events of the last 32 calls are kept.  fc_get_kernel_times
 * waits for those calls and writes, for each kernel, its elapsed milliseconds
 * averaged over the calls made since profiling was switched on (at most the
 * last 32; 0 if it was never launched) to host_ms[0..FC_N_KERNELS).
 * fc_kernel_name(i) names slot i.  fc_set_profiling(pool, 1) restarts the
 * average.
 */
#define FC_N_KERNELS 11
int fc_set_profiling(fc_pool* pool, int enable);
int fc_get_kernel_times(fc_pool* pool, float* host_ms);
const char* fc_kernel_name(int i);

/* Text of the most recent error raised on the calling thread ("" if none). */
const char* fc_last_error(void);

/*
 * Decode-side pool traffic (Algorithm 1, ExecuteDecoding: every decode step
 * reads the compressed cache of each request, M.Generate, and appends the new
 * token's K and V, UpdateKVCache).
 *
 * fc_append_batch: for every request r (with host_enable[r] != 0 if
 * host_enable is given) the new token's rows dev_new_kv[r] go to token
 * position L_r = host_seq_lens[r]: slot L_r % 16 of the block in table entry
 * L_r / 16.  When L_r is a multiple of 16 a block is popped first (requests
 * in batch order) and written to that table entry.  host_seq_lens[r] becomes
 * L_r + 1 before the call returns; the device work is asynchronous on stream.
 *   dev_new_kv  dev, fp16 [n_req][n_layers][2][n_heads][head_dim], 16-byte aligned
 * FC_EINVAL: L_r < 0 or >= FC_MAX_SEQ_LEN, table row full (L_r/16 >=
 * max_blocks_per_req); FC_ENOMEM: more blocks needed than are free.  Nothing
 * is modified on error.
 *
 * fc_decode_attention: the single-query attention of one decode step over
 * the paged cache, for every request, layer and head:
 *   out = softmax(scale * K q) . V   over the request's L_r cached tokens
 * (fp16 K, V, q; fp32 arithmetic; zeros for L_r = 0; scale <= 0 means
 * 1/sqrt(head_dim)).  Reads every cached K and V row once.
 *   dev_q    dev, fp16 [n_req][n_layers][n_heads][head_dim], 16-byte aligned
 *   dev_out  dev, fp32 [n_req][n_layers][n_heads][head_dim]
 */
int fc_append_batch(fc_pool* pool, int32_t* dev_block_tables, int max_blocks_per_req,
                    int32_t* host_seq_lens, const void* dev_new_kv, const int32_t* host_enable,
                    int n_req, void* stream);
int fc_decode_attention(fc_pool* pool, const int32_t* dev_block_tables, int max_blocks_per_req,
                        const int32_t* host_seq_lens, const void* dev_q, float* dev_out,
                        int n_req, float scale, void* stream);

/*
 * The same attention over a cache that was pruned but NOT compacted (tokens
 * evicted in place leave holes, so no block can be returned to the pool and
 * every kept row is read from where it lies): request r, layer l, head h
 * attends over the host_budget[r] tokens listed, in ascending order, in
 *   dev_kept   dev, int32, packed [r][layer][head][host_budget[r]] in batch
 *              order (the layout of fc_compress_batch's dev_kept_out),
 * read through the request's UNCOMPRESSED block table and length.  It is the
 * counterfactual that the compaction copy of the stage is measured against
 * (same result as fc_decode_attention on the compacted cache); indices outside
 * 0..L_r-1 are clamped.  FC_EINVAL additionally for a budget outside 0..L_r.
 */
int fc_decode_attention_kept(fc_pool* pool, const int32_t* dev_block_tables,
                             int max_blocks_per_req, const int32_t* host_seq_lens,
                             const int32_t* host_budget, const int32_t* dev_kept,
                             const void* dev_q, float* dev_out, int n_req, float scale,
                             void* stream);

/*
 * Host-side scheduler of the compress queue (Algorithm 1, ServeRequests:
 * AccumulateRequests, the |Q| >= B_min / WaitTimeExceeded test, FormBatch(Q,
 * B_max), AdjustBatch; "Memory-Aware Scheduling" paragraph: all pending
 * requests are examined and the largest batch that fits the free memory is
 * built, not the head of the queue).  Pure host code, no device work: the
 * caller passes fc_pool_num_free() and hands the batch to fc_compress_batch.
 * Times are integer microseconds on any clock of the caller's.
 *
 *  - a request needs ceil(budget/16) free blocks in the compress stage;
 *  - the trigger fires when requests are pending and (their number >= the
 *    current batch target, which starts at b_min, or the oldest has waited
 *    max_wait_us or longer);
 *  - fc_sched_form_batch: 0 if the trigger has not fired; else requests whose
 *    wait time is exceeded are taken first, in arrival order, each if it
 *    still fits (free blocks, b_max, capacity) and skipped if not; then the
 *    others in order of (need, arrival, id) while they fit.  The ids are
 *    written to out_ids (host, capacity entries) in arrival order, the
 *    requests leave the queue, the return value is their number (0 if nothing
 *    fits).
 *  - fc_sched_adjust(service_us): report how long the last batch took; the
 *    batch target becomes ceil(service / gap) clamped to [b_min, b_max],
 *    with running averages avg += floor((x - avg)/4) (first sample sets avg)
 *    of the service times and of the gaps between arrivals; returns it.
 * fc_sched_submit: FC_EINVAL (nothing changed) for an arrival before the last
 * one, a budget outside 1..seq_len, or an id that is still pending.
 */
typedef struct fc_sched fc_sched;
int fc_sched_create(fc_sched** out, int b_min, int b_max, int64_t max_wait_us);
void fc_sched_destroy(fc_sched* sched);
int fc_sched_submit(fc_sched* sched, int64_t req_id, int64_t arrival_us, int seq_len, int budget);
int fc_sched_pending(const fc_sched* sched);
int fc_sched_batch_target(const fc_sched* sched);
int fc_sched_ready(const fc_sched* sched, int64_t now_us);
int fc_sched_form_batch(fc_sched* sched, int64_t now_us, int free_blocks, int64_t* out_ids,
                        int capacity);
int fc_sched_adjust(fc_sched* sched, int64_t service_us);

#ifdef __cplusplus
}
#endif
#endif /* FASTCACHE_H */
