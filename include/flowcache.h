/*
 * flowcache.h -- C ABI of the FlowCache denoising-step hot path for AMD MI355X (gfx950).
 *
 * The library implements, as hand-written HIP kernels, the per-tick work that FlowCache
 * ("Flow Caching for Autoregressive Video Generation") adds to, or keeps from, a causal
 * diffusion-forcing video DiT layer:
 *
 *   flowcache_chunk_decide    per-chunk relative-L1 change metric, accumulate-and-threshold
 *                             reuse decision and gather of the chunks to recompute
 *                             (Sec. 3.2, Eq. (5) and Eq. (8)).
 *   flowcache_uniform_decide  the uniform ("traditional reuse") policy the paper compares with:
 *                             one shared accumulator and decision for all chunks past
 *                             warm-up (Fig. 2, top).
 *   flowcache_residual_apply  cached-activation reuse around the skipped forward pass:
 *                             recompute chunks store (output - input), reused chunks get
 *                             input + stored difference; compact -> full layout (Sec. 3.2).
 *   flowcache_attend          chunk-causal multi-head attention of the recompute chunks
 *                             against [clean KV cache | active chunks' KV], optionally
 *                             emitting the per-key attention mass (Sec. 3.3, Eq. (9)).
 *   flowcache_scatter_kv      new K/V of the recompute chunks into their cache slots (the
 *                             scatter half of the gather step; Sec. 3.2).
 *   flowcache_attention_mass  the importance mass alone, for explicit observation queries
 *                             (Sec. 3.3, Eq. (9); observation window of App. C.2).
 *   flowcache_kv_compress     joint importance-redundancy scoring, per-head top-B selection
 *                             and in-place compaction of K and V (Sec. 3.3, Eq. (10)-(12),
 *                             linear-time redundancy of App. C.2, phases of App. C.1).
 *   flowcache_kv_select,
 *   flowcache_kv_compact      the two halves of flowcache_kv_compress as calls of their own.
 *   flowcache_kv_compress_grouped  the same at frame / chunk key granularity (App. D.2.1).
 *
 * Conventions common to all calls
 * -------------------------------
 *  - Pointers marked [dev] are DEVICE pointers owned by the caller; [host] are host
 *    pointers read during the call only.  The library never allocates, frees or keeps a
 *    pointer.  Scratch space is a caller-provided device workspace whose size comes from
 *    the matching *_workspace() query (256-byte aligned; contents need no initialisation
 *    and are undefined afterwards).
 *  - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default
 *    stream) and the call returns without synchronising.  Calls that share a workspace
 *    must be stream-ordered.
 *  - Return value: FC_OK or an error code.  Argument errors are detected and returned
 *    BEFORE any HIP call is made, so they can be exercised on a machine without a GPU.
 *    No exception crosses the boundary; the library keeps no state between calls (except the
 *    device address of its own scratch buffer, see flowcache_chunk_decide_noalloc).
 *  - dtype FC_F32: float tensors, fp32 arithmetic.  FC_BF16: bfloat16 tensors, bf16 x bf16
 *    -> fp32 matrix-core products, fp32 softmax state, bf16 output.
 *  - The recompute list (recompute_idx, n_recompute) lives on the device, so the host
 *    cannot check it: the kernels do.  A count above A is cut to A and an entry outside
 *    [0, A) is skipped (nothing is read or written for it); no out-of-range access follows
 *    from a bad list.
 *  - Decisions (reuse masks) and kept-token indices are taken in float64 and are meant to
 *    be bit-reproducible run to run: no floating-point atomics are used anywhere.
 */
#ifndef FLOWCACHE_H
#define FLOWCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { FC_F32 = 0, FC_BF16 = 1 } fc_dtype;

typedef void* fc_stream; /* hipStream_t */

enum {
    FC_OK = 0,
    FC_INVALID_ARGUMENT = 1,    /* null pointer, negative size, eps < 0 or NaN, even pool width ... */
    FC_UNSUPPORTED = 2,         /* shape/dtype outside what the kernels cover (e.g. head_dim)       */
    FC_WORKSPACE_TOO_SMALL = 3, /* workspace_bytes below the *_workspace() figure                   */
    FC_HIP_ERROR = 4            /* a HIP runtime call or kernel launch failed                       */
};

#define FC_MAX_ACTIVE 16 /* largest number of active chunks in the denoising window */

/* Human-readable name of a status code (static storage). */
const char* flowcache_status_string(int status);

/* Library version, major*100 + minor. */
int flowcache_version(void);

/*
 * Change metric, reuse decision and gather.  Sec. 3.2: Eq. (5) per chunk, then Eq. (8).
 *
 *   L1rel_i = sum|x_cur[i] - x_prev[i]| / sum|x_prev[i]|        (previous tick in the denominator;
 *                                                                  zero denominator -> +inf)
 *   step_idx[i] < warmup_m          : f_i = 0                    (first m local steps never reuse)
 *   acc[i] + L1rel_i  > eps         : f_i = 0
 *   otherwise                       : f_i = acc[i] + L1rel_i
 *   recompute_i = (f_i == 0);  acc[i] <- f_i
 *
 * Elements are widened exactly to float64; sums and the comparison are float64.
 *
 *   x_cur, x_prev  [dev] [A, chunk_elems] contiguous, `dtype`
 *   step_idx       [dev] [A] int32, steps already taken by each chunk
 *   acc            [dev] [A] float64, in/out accumulator f
 *   l1rel          [dev] [A] float64 out, may be NULL
 *   recompute_mask [dev] [A] uint8 out, 1 = recompute
 *   recompute_idx  [dev] [A] int32 out: ascending list of chunks to recompute in its first
 *                        *n_recompute entries, the rest set to -1
 *   n_recompute    [dev] [1] int32 out
 *   x_compact      [dev] [A, chunk_elems] out, may be NULL: block r receives
 *                        x_cur[recompute_idx[r]] for r < *n_recompute; other blocks untouched
 * Errors: A outside [1, FC_MAX_ACTIVE], chunk_elems < 1, warmup_m < 0, eps < 0 or not
 * finite, null pointers -> FC_INVALID_ARGUMENT.
 */
int flowcache_chunk_decide(const void* x_cur, const void* x_prev, fc_dtype dtype, int A,
                           int64_t chunk_elems, const int32_t* step_idx, int warmup_m,
                           double eps, double* acc, double* l1rel, uint8_t* recompute_mask,
                           int32_t* recompute_idx, int32_t* n_recompute, void* x_compact,
                           void* workspace, size_t workspace_bytes, fc_stream stream);
size_t flowcache_chunk_decide_workspace(int A, int64_t chunk_elems);

/*
 * flowcache_chunk_decide for callers that cannot allocate device memory and have no workspace
 * to hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments (minus the workspace), same kernels and bit-identical results.
 * The block partials go to a buffer of FC_DECIDE_SCRATCH_BYTES that the library itself holds
 * in device memory (one per GPU, for the life of the process).  The call allocates and frees
 * nothing, enqueues on `stream` and returns without synchronising.
 *   - Every call on a GPU shares that GPU's buffer: calls that may overlap on one GPU (two
 *     streams, two threads) race and must be ordered by the caller.  Nothing in the buffer has
 *     to survive between calls and nothing in it has to start at zero.
 *   - A launch whose partials would not fit (flowcache_chunk_decide_workspace(A, chunk_elems) >
 *     FC_DECIDE_SCRATCH_BYTES) is rejected with FC_WORKSPACE_TOO_SMALL before any HIP call;
 *     with A <= FC_MAX_ACTIVE the launches of this version never need more than 32 KiB.
 *   - FC_HIP_ERROR if the buffer's address cannot be obtained on the current device.
 */
#define FC_DECIDE_SCRATCH_BYTES 32768
int flowcache_chunk_decide_noalloc(const void* x_cur, const void* x_prev, fc_dtype dtype, int A,
                                   int64_t chunk_elems, const int32_t* step_idx, int warmup_m,
                                   double eps, double* acc, double* l1rel,
                                   uint8_t* recompute_mask, int32_t* recompute_idx,
                                   int32_t* n_recompute, void* x_compact, fc_stream stream);

/*
 * Uniform reuse policy (Fig. 2, top: the policy the chunkwise one is compared with): the relative L1
 * change is taken over ALL chunks past warm-up together,
 *
 *   L1rel = sum_{i: step_idx[i] >= m} sum|x_cur[i] - x_prev[i]| / sum_{i: ...} sum|x_prev[i]|,
 *   a = acc_global + L1rel;  f = (a > eps) ? 0 : a;  acc_global <- f,
 *
 * every such chunk recomputes iff f == 0, and a chunk still in warm-up always recomputes.
 * With no chunk past warm-up acc_global is reset to 0 and *l1rel is NaN.
 * Arguments as for flowcache_chunk_decide except
 *   acc_global [dev] [1] float64 in/out,   l1rel [dev] [1] float64 out, may be NULL.
 * Uses the same workspace size as flowcache_chunk_decide.
 */
int flowcache_uniform_decide(const void* x_cur, const void* x_prev, fc_dtype dtype, int A,
                             int64_t chunk_elems, const int32_t* step_idx, int warmup_m,
                             double eps, double* acc_global, double* l1rel,
                             uint8_t* recompute_mask, int32_t* recompute_idx,
                             int32_t* n_recompute, void* x_compact, void* workspace,
                             size_t workspace_bytes, fc_stream stream);

/*
 * Cached-activation reuse (Sec. 3.2: when f != 0 the cached activations are reused instead
 * of the forward pass).  The cache holds, per active chunk, the difference between the
 * stack's output and its input at the chunk's last recompute:
 *
 *   chunk c = recompute_idx[r], r < *n_recompute:  residual[c] <- y_compact[r] - x_cur[c]
 *                                                  out[c]      <- y_compact[r]
 *   any other chunk c:                             out[c]      <- x_cur[c] + residual[c]
 *
 * Operands are widened exactly to float64, the sum or difference is taken in float64 and
 * rounded ONCE (to nearest even) to `dtype`.
 *
 *   x_cur      [dev] [A, chunk_elems] input of the stack this tick
 *   y_compact  [dev] [A, chunk_elems] compact: block r = output for chunk recompute_idx[r]
 *                    (blocks r >= *n_recompute are not read); may be NULL when nothing is
 *                    recomputed this tick: then the list is not consulted and every chunk
 *                    is treated as reused
 *   residual   [dev] [A, chunk_elems] in/out cache
 *   out        [dev] [A, chunk_elems] full-layout output of the stack; may alias x_cur
 *   recompute_idx, n_recompute [dev] as written by the decide calls
 * Errors: null pointers (except y_compact), A outside [1, FC_MAX_ACTIVE], chunk_elems < 1
 * -> FC_INVALID_ARGUMENT.
 */
int flowcache_residual_apply(const void* x_cur, const void* y_compact, void* residual, void* out,
                             fc_dtype dtype, int A, int64_t chunk_elems,
                             const int32_t* recompute_idx, const int32_t* n_recompute,
                             fc_stream stream);

/*
 * Chunk-causal attention of the recompute chunks.  Sec. 3.3 (clean chunks live in the KV
 * cache and are attended by the chunks being denoised); softmax(q K^T * scale) V.
 *
 * A query of active chunk c sees cache positions [0, L_clean) and the slots of active
 * chunks 0..c (its own chunk entirely: bidirectional inside a chunk, causal across chunks).
 * Slots of chunks that are NOT recomputed this tick keep, and expose, their stale K/V.
 *
 *   q        [dev] [A*L_c, H_q, d] compact: row block r <-> chunk recompute_idx[r]
 *   k_new,
 *   v_new    [dev] [A*L_c, H_k, d] compact, same row blocks; may both be NULL when the
 *                  caller has already written the slots.  Otherwise block r is first
 *                  copied into slot active_off[recompute_idx[r]] of the caches.
 *   k_cache,
 *   v_cache  [dev] head-major: element (h, pos, e) at h*kv_head_stride + pos*kv_tok_stride + e
 *                  (strides in elements; d <= kv_tok_stride <= 2^24 and a multiple of 8,
 *                  kv_head_stride >= capacity*kv_tok_stride)
 *   capacity       number of token positions per head in the caches
 *   active_off [host] [A] first cache position of each active chunk's slot, in causal
 *                  order; slots are L_c long, lie in [L_clean, capacity] and do not overlap
 *   recompute_idx, n_recompute [dev] as written by flowcache_chunk_decide
 *   softmax_scale  0 selects d^-1/2
 *   out      [dev] [A*L_c, H_q, d] `dtype`; only row blocks r < *n_recompute are written
 *   lse      [dev] [H_q, A*L_c] float32 natural-log sum-exp of each row, may be NULL
 *   mass     [dev] [H_k, mass_len] float32, may be NULL.  When given, receives Eq. (9)
 *                  over cache positions [0, mass_len): the mean, over the last `obs_window`
 *                  rows (0 = all L_c rows) of the LAST compact row block and over the
 *                  H_q/H_k query heads of each key head, of softmax restricted to those
 *                  positions.  That block must hold the last active chunk (A-1); if it
 *                  does not, mass is filled with NaN.
 * Supported: d in {64, 128}; H_q % H_k == 0; A <= FC_MAX_ACTIVE; FC_BF16 needs d == 128 or 64.
 */
int flowcache_attend(const void* q, const void* k_new, const void* v_new, void* k_cache,
                     void* v_cache, int64_t kv_head_stride, int64_t kv_tok_stride,
                     int capacity, fc_dtype dtype, int H_q, int H_k, int d, int L_c,
                     int L_clean, int A, const int32_t* active_off,
                     const int32_t* recompute_idx, const int32_t* n_recompute,
                     float softmax_scale, void* out, float* lse, float* mass, int mass_len,
                     int obs_window, void* workspace, size_t workspace_bytes,
                     fc_stream stream);
size_t flowcache_attend_workspace(int A, int L_c, int H_q, int H_k, int d, int mass_len,
                                  int obs_window);

/*
 * The K/V half of the gather/scatter step on its own (flowcache_attend performs it when
 * k_new/v_new are given): block r < *n_recompute of the compact token-major k_new/v_new
 * ([A*L_c, H_k, d]) is copied into slot active_off[recompute_idx[r]] of the head-major
 * caches.  Sec. 3.2 (only the chunks chosen for recomputation produce new K/V); slots of
 * reused chunks are not touched.  Arguments as in flowcache_attend.
 */
int flowcache_scatter_kv(const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                         int64_t kv_head_stride, int64_t kv_tok_stride, int capacity,
                         fc_dtype dtype, int H_k, int d, int L_c, int L_clean, int A,
                         const int32_t* active_off, const int32_t* recompute_idx,
                         const int32_t* n_recompute, fc_stream stream);

/*
 * Importance mass, Eq. (9), for explicit observation queries (App. C.2 uses the last 50
 * query tokens of the last denoising chunk).
 *
 *   q_obs  [dev] [W, H_q, d] `dtype`
 *   k_cache [dev] head-major as above; positions [0, mass_len) are scored
 *   mass   [dev] [H_k, mass_len] float32 out; each row sums to 1
 */
int flowcache_attention_mass(const void* q_obs, int W, const void* k_cache,
                             int64_t kv_head_stride, int64_t kv_tok_stride, fc_dtype dtype,
                             int H_q, int H_k, int d, int mass_len, float softmax_scale,
                             float* mass, void* workspace, size_t workspace_bytes,
                             fc_stream stream);
size_t flowcache_attention_mass_workspace(int W, int H_q, int H_k, int d, int mass_len);

/*
 * KV-cache compression at a chunk commit.  Sec. 3.3, per key head h over the first L_k
 * cache positions (the merged set: clean region followed by the chunk that just finished):
 *
 *   Imp~_j  = max of mass over the window |u - j| <= pool_k/2                      Eq. (10)
 *   k^_j    = k_j / max(||k_j||_2, 1e-12)
 *   r_j     = (k^_j . sum_i k^_i  -  k^_j . k^_j) / L_k     linear form, App. C.2, of the
 *                                                           diagonal-zeroed mean of Eq. (11)
 *   Red_j   = softmax_j(r)                                                         Eq. (11)
 *   Score_j = lambda * Imp~_j - (1 - lambda) * Red_j                               Eq. (12)
 *
 * The `budget` highest scores are kept (ties: lower position wins); the kept rows of K
 * and V move, in ascending original position, to positions [0, budget) of the same buffers.
 * Positions >= budget keep their old contents.  budget >= L_k is the cache-filling phase
 * of App. C.1: kept_idx = 0..L_k-1 and the buffers are untouched.  All scoring arithmetic
 * is float64.
 *
 *   mass     [dev] [H_k, L_k] float32, Eq. (9) importance before pooling
 *   kept_idx [dev] [H_k, min(budget, L_k)] int32 out, ascending original positions
 * Errors: pool_k even or < 1, lambda outside [0,1], budget < 1, L_k < 1 -> FC_INVALID_ARGUMENT;
 * d not in {64, 128} -> FC_UNSUPPORTED.
 */
int flowcache_kv_compress(void* k_cache, void* v_cache, int64_t kv_head_stride,
                          int64_t kv_tok_stride, fc_dtype dtype, int H_k, int d, int L_k,
                          int budget, const float* mass, int pool_k, double lambda,
                          int32_t* kept_idx, void* workspace, size_t workspace_bytes,
                          fc_stream stream);
size_t flowcache_kv_compress_workspace(int H_k, int L_k, int d, int budget, fc_dtype dtype);

/*
 * The two halves of flowcache_kv_compress as calls of their own, for callers that overlap the
 * scoring and selection (which only read K) with other work on another stream -- the
 * attention of the same tick, say -- and move the rows afterwards.  Same arguments, same
 * workspace size (flowcache_kv_compress_workspace) and same results: select followed by
 * compact leaves kept_idx, K and V bit-identical to one flowcache_kv_compress call
 * (Sec. 3.3, Eq. (10)-(12) for the first; the in-place compaction for the second).
 *
 *   flowcache_kv_select   writes kept_idx [H_k, min(budget, L_k)]; K is not modified
 *   flowcache_kv_compact  moves row kept_idx[h][i] of K and V to position i, for i < budget
 *                         (nothing moves when budget >= L_k).  kept_idx [dev] must be
 *                         ascending per head, as written by flowcache_kv_select; entries
 *                         outside [0, L_k) are skipped.  The status word of
 *                         flowcache_kv_compress_status_offset applies to this call too.
 */
int flowcache_kv_select(const void* k_cache, int64_t kv_head_stride, int64_t kv_tok_stride,
                        fc_dtype dtype, int H_k, int d, int L_k, int budget, const float* mass,
                        int pool_k, double lambda, int32_t* kept_idx, void* workspace,
                        size_t workspace_bytes, fc_stream stream);
int flowcache_kv_compact(void* k_cache, void* v_cache, int64_t kv_head_stride,
                         int64_t kv_tok_stride, fc_dtype dtype, int H_k, int d, int L_k,
                         int budget, const int32_t* kept_idx, void* workspace,
                         size_t workspace_bytes, fc_stream stream);

/*
 * The same compression with keys scored and kept at a coarser granularity (the frame- and
 * chunk-level key granularities of the ablation in App. D.2.1).  The first L_k positions
 * are split into groups of `group` consecutive tokens (a latent frame, or a chunk).  A group
 * is represented by the mean of its keys and the mean of its tokens' mass (float64 sums and
 * means, kept as float64); Eq. (10)-(12) and the top-B selection run over the groups exactly
 * as they run over tokens in flowcache_kv_compress; every token of a kept group is kept.
 *
 *   group    tokens per group, >= 1 (1 = flowcache_kv_compress); L_k and budget (both in
 *            tokens) must be multiples of it
 *   pool_k   window of Eq. (10), counted in groups
 *   kept_idx [dev] [H_k, min(budget, L_k)] int32 out: kept TOKEN positions, ascending
 * Errors as for flowcache_kv_compress, plus FC_INVALID_ARGUMENT when L_k or budget is not a
 * multiple of group.
 */
int flowcache_kv_compress_grouped(void* k_cache, void* v_cache, int64_t kv_head_stride,
                                  int64_t kv_tok_stride, fc_dtype dtype, int H_k, int d, int L_k,
                                  int budget, int group, const float* mass, int pool_k,
                                  double lambda, int32_t* kept_idx, void* workspace,
                                  size_t workspace_bytes, fc_stream stream);
size_t flowcache_kv_compress_grouped_workspace(int H_k, int L_k, int d, int budget, int group,
                                               fc_dtype dtype);

/*
 * The in-place compaction orders its row tiles with bounded waits (a tile stores only after
 * the lower tiles that still read its rows have loaded them).  Should such a wait ever run
 * into its spin limit the kernel does not hang: it sets a status word in the workspace.  This
 * returns the BYTE OFFSET of that uint32 inside the workspace of a compress call with the same
 * arguments (group = 1 for flowcache_kv_compress): 0 after the call = all waits were served,
 * non-zero = the contents of the caches are unspecified.  Only meaningful when budget < L_k
 * (the identity case does not touch the workspace).  (size_t)-1 for invalid arguments.
 */
size_t flowcache_kv_compress_status_offset(int H_k, int L_k, int d, int budget, int group,
                                           fc_dtype dtype);

#ifdef __cplusplus
}
#endif
#endif /* FLOWCACHE_H */
