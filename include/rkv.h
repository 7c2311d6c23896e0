/*
 * rkv.h — C ABI of the R-KV decode-time KV-cache compression step for AMD MI355X (gfx950).
 *
 * The step runs in every layer each time the decode buffer fills (Sec. 3.1): of the
 * N = B_budget + B_buffer cached tokens the last `alpha` (observation tokens) are always
 * kept, the first n = N - alpha are candidates, and k = budget - alpha candidates are
 * selected per KV head by the joint score of Sec. 3.4.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library never
 *     allocates, frees or keeps them.  `rkv_params` and `size_t*` are HOST pointers.
 *   - bf16 tensors are row-major with the head dimension innermost and contiguous:
 *       q_obs [P, q_heads, alpha, d]   observation queries; query head hq serves KV head
 *                                      hq / G, G = q_heads / kv_heads (Sec. 3.2, GQA); strides in
 *                                      `rkv_params` (e.g. a query cache laid out [P, alpha, q_heads, d])
 *       k, v  [P, kv_heads, N, d]      token order = row order; strides in `rkv_params`
 *     fp32 / int32 outputs are dense: [P, kv_heads, n] or [P, kv_heads, budget].
 *   - P = num_problems independent (sequence, layer) pairs are processed per call.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream)
 *     and the call returns without synchronising the device.
 *   - `ws` is caller-provided device scratch of at least rkv_workspace_size() bytes,
 *     256-byte aligned; contents need not be preserved between calls.
 *   - Errors are returned as negative rkv_status values.  Arguments are validated before the
 *     first launch: for every negative status except RKV_ERR_HIP nothing has been enqueued and
 *     the outputs are untouched (after RKV_ERR_HIP earlier stages of the call may have run).
 *   - Inputs holding NaN or Inf give unspecified scores (never out-of-bounds accesses).
 *   - Supported shapes: d == 128, 1 <= alpha <= 64, G * alpha <= 64, N <= 32768,
 *     pool_w <= 1000 and alpha * 2 * pool_w <= 16384,
 *     token strides multiples of 8 elements (16-byte aligned rows).
 *   - Paged caches (optional): with page_size > 0 the k and v pointers are the bases of page pools
 *     and token t of problem p lives in page block_table[p * table_stride + t / page_size] at slot
 *     t % page_size:  element offset = page * k_stride_page + h * k_stride_head + slot * k_stride_token
 *     (likewise v).  page_size is 16, 32, 64 or 128; k_stride_problem / v_stride_problem are ignored.
 *     Every entry point that reads or writes k, v accepts this layout; k_out / v_out of rkv_compact
 *     and rkv_compress are never paged.  The workspace then also holds a dense copy of the candidate
 *     keys (written by the pre-pass on its single read of K, read by the similarity pass).
 */
#ifndef RKV_H
#define RKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  RKV_OK = 0,
  RKV_NOT_TRIGGERED = 1,     /* N <= budget: nothing to evict, nothing enqueued (the early returns of Alg. 1) */
  RKV_ERR_NULL = -1,         /* a required pointer is NULL */
  RKV_ERR_SHAPE = -2,        /* inconsistent sizes: q_heads % kv_heads, budget <= alpha, N <= alpha, strides */
  RKV_ERR_UNSUPPORTED = -3,  /* outside the supported shapes listed above, or unknown flag bits */
  RKV_ERR_WORKSPACE = -4,    /* ws is NULL, misaligned or smaller than rkv_workspace_size() */
  RKV_ERR_PARAM = -5,        /* lambda or sim_threshold outside [0, 1], beta < 0, eps <= 0, pool_w < 0 */
  RKV_ERR_HIP = -6           /* a kernel launch failed (hipGetLastError) */
} rkv_status;

/*
 * rkv_params.flags.  RKV_FLAG_SKIP_SATURATED: exact shortcut of the redundancy pass.  A token whose
 * `beta` most recent similar tokens have been found cannot change any more (Sec. 3.3 zeroes only those
 * beta entries), so rows in that state take no further part in the pass and the rows still open are
 * gathered into fewer waves as their number falls.  Results are bit-identical to flags = 0; only the
 * amount of matrix work differs (data dependent).
 */
#define RKV_FLAG_SKIP_SATURATED 1u
/*
 * Two variants that follow the paper's pseudo-code (Alg. 1) where it differs from the equations.
 * RKV_FLAG_POOL_AFTER_MEAN: the attention weights are averaged over the alpha query rows first and the
 * 2W-wide sliding max is applied to that average (default, Eq. 4: pool every row, then average).
 * Needs (alpha + 1) * 2W <= 16384.
 * RKV_FLAG_SHARED_SELECTION: the per-head scores Z are averaged over the H KV heads of a problem and
 * the budget - alpha candidates with the largest average are kept in every head (default, Sec. 3.4:
 * each head selects by its own Z).  kept_idx[p, h, :] is then the same list for every h; `score`
 * still receives the per-head Z.  Applies to rkv_select_topk and rkv_compress.
 */
#define RKV_FLAG_POOL_AFTER_MEAN 2u
#define RKV_FLAG_SHARED_SELECTION 4u
/*
 * How the G query heads of a group are merged.  Default (Eq. 2-3 as printed): element-wise max of the raw
 * scaled logits, then one softmax over the candidates.  App. A.2 describes the pooling as acting on
 * attention scores: RKV_FLAG_GQA_SOFTMAX_THEN_MAX takes the softmax of every query head and then the max
 * over the group (not renormalised), RKV_FLAG_GQA_SOFTMAX_THEN_MEAN the mean over the group (the pooling
 * App. A.2 attributes to earlier work).  The two are mutually exclusive (RKV_ERR_PARAM); both make the
 * workspace hold G * alpha instead of alpha logit rows per head.
 */
#define RKV_FLAG_GQA_SOFTMAX_THEN_MAX 8u
#define RKV_FLAG_GQA_SOFTMAX_THEN_MEAN 16u
/*
 * Direction of the keep-recent rule of Sec. 3.3.  Default (what the text and Alg. 1 both spell out): the
 * similarity of token i to each of its beta most recent similar tokens j is dropped from token i's own
 * average.  RKV_FLAG_RECENCY_TRANSPOSED drops it from the recent partner j's average instead, which is
 * what the stated purpose (keep the most recent of a group of similar tokens) suggests: among exact
 * copies the newest then has the lowest redundancy.  Needs 8 more workspace bytes per candidate.
 */
#define RKV_FLAG_RECENCY_TRANSPOSED 32u
/*
 * RKV_FLAG_TRIANGULAR_SCAN: another schedule of the redundancy pass for the default rule with beta = 1, same
 * result up to the order of a few floating-point operations.  The cosine matrix of Eq. 5 is symmetric, so
 * only the entries with j < i are formed (by row blocks: about two thirds of the matrix work at the
 * benchmark sizes, tending to one half for long caches); an entry above T is the most recent partner
 * candidate of token i among the older tokens and, mirrored, a newer partner of token j, which a 64-bit
 * atomic maximum per token collects.  A row cannot be left alone after its first partner (its later entries
 * may be some older token's most recent partner), so every tile that holds an entry above T takes the slow
 * path: the mode pays only where such entries are rare (high T, little redundancy).  Needs beta == 1 and
 * neither RKV_FLAG_RECENCY_TRANSPOSED nor RKV_FLAG_SKIP_SATURATED (RKV_ERR_PARAM otherwise) and 16 more
 * workspace bytes per candidate.
 */
#define RKV_FLAG_TRIANGULAR_SCAN 64u

typedef struct {
  int32_t num_problems;      /* P >= 0; an empty batch is valid and enqueues nothing */
  int32_t kv_heads;          /* H */
  int32_t q_heads;           /* H * G */
  int32_t n_tokens;          /* N = rows currently held per head (budget + buffer) */
  int32_t head_dim;          /* d = 128 */
  int32_t alpha;             /* observation window (paper: 8) */
  int32_t budget;            /* rows kept per head = (budget - alpha) selected + alpha observation rows */
  int32_t pool_w;            /* W of the 2W-wide max-pool window [i-W, i+W-1] (Eq. 4); 0 = no pooling */
  int32_t beta;              /* most recent similar tokens whose similarity is zeroed (Sec. 3.3) */
  float   sim_threshold;     /* T, strict '>' (Sec. 3.3) */
  float   lambda;            /* trade-off of Eq. 7 (paper: 0.1) */
  float   eps;               /* added to the key norm (Eq. 5, paper: 1e-8); must be > 0, which is what keeps an
                                all-zero key row finite (its similarities are then 0) */
  uint32_t flags;            /* 0 or RKV_FLAG_* bits */
  int64_t k_stride_problem, k_stride_head, k_stride_token;   /* in elements; 0,0,0 = dense [P,H,N,d] */
  int64_t v_stride_problem, v_stride_head, v_stride_token;   /* in elements; 0,0,0 = dense [P,H,N,d] */
  int64_t o_stride_problem, o_stride_head, o_stride_token;   /* of k_out and v_out; 0,0,0 = dense [P,H,budget,d] */
  int64_t q_stride_problem, q_stride_head, q_stride_token;   /* of q_obs / the query cache, in elements: problem, query
                                                                head, window slot; 0,0,0 = dense [P,q_heads,alpha,d] */
  int32_t page_size;         /* 0 = contiguous caches; 16, 32, 64 or 128 tokens per page otherwise */
  int32_t table_stride;      /* entries of block_table per problem, >= ceil(N / page_size) */
  const int32_t* block_table;/* DEVICE pointer, int32 [P, table_stride] page indices (paged caches only) */
  int64_t k_stride_page, v_stride_page;                      /* in elements (paged caches only) */
} rkv_params;

/* Bytes of device scratch any entry point below needs for these params. */
rkv_status rkv_workspace_size(const rkv_params* prm, size_t* bytes);

/*
 * Importance score, Sec. 3.2: scaled logits of the G query heads of each KV head against the
 * n candidate keys (Eq. 2), element-wise max over the group, softmax over the candidates
 * (Eq. 3; Eq. 1 when G = 1), 2W-wide sliding max per query row and mean over the alpha rows
 * (Eq. 4).  Writes importance[P, H, n] (fp32).  `v` strides are ignored.
 */
rkv_status rkv_score_importance(const rkv_params* prm, const void* q_obs, const void* k,
                                float* importance, void* ws, size_t ws_bytes, void* stream);

/*
 * Redundancy score, Sec. 3.3: cosine similarity of the candidate keys with eps added to each
 * norm and a zero diagonal (Eq. 5); for every token the similarities above T to its `beta`
 * most recent (largest-index) similar tokens are zeroed; row average over n and softmax over
 * the candidates (Eq. 6).  Writes redundancy[P, H, n]; if mean_sim is not NULL also the
 * averages before the softmax, [P, H, n].  The n x n matrix is never stored.
 */
rkv_status rkv_score_redundancy(const rkv_params* prm, const void* k, float* redundancy,
                                float* mean_sim, void* ws, size_t ws_bytes, void* stream);

/*
 * Joint score and selection, Sec. 3.4 and 3.1: Z = lambda * I - (1 - lambda) * R (Eq. 7); per
 * head the k = budget - alpha candidates with the largest Z are kept (equal Z: the larger index
 * wins).  kept_idx[P, H, budget] (int32) receives the kept candidates in ascending order followed
 * by the observation rows n .. N-1.  If score is not NULL it receives Z[P, H, n].
 */
rkv_status rkv_select_topk(const rkv_params* prm, const float* importance, const float* redundancy,
                           float* score, int32_t* kept_idx, void* ws, size_t ws_bytes, void* stream);

/*
 * Compaction (Alg. 1, gather + concatenate): k_out[p, h, r, :] = k[p, h, kept_idx[p, h, r], :],
 * likewise v.  k_out, v_out are [P, H, budget, d] bf16 (dense unless o_stride_* are set, e.g. to write
 * into the first `budget` rows of a second cache allocation) and must not overlap k, v.
 * Every index must lie in [0, N); indices outside are clamped into that range.
 */
rkv_status rkv_compact(const rkv_params* prm, const void* k, const void* v, const int32_t* kept_idx,
                       void* k_out, void* v_out, void* stream);

/*
 * Compaction in place (Alg. 1 keeps one cache and sets its length to the budget): afterwards rows
 * 0 .. budget-1 of k[p, h] and v[p, h] hold the rows kept_idx[p, h, :] selected; rows budget .. N-1 are
 * left as they were.  kept_idx[P, H, budget] must be strictly ascending per head (as rkv_select_topk
 * and rkv_compress write it), which makes every row move towards the front; a list that is not gives
 * unspecified row contents (indices are still clamped into [0, N), nothing is accessed out of bounds).
 * k, v use k_stride_* / v_stride_*; o_stride_* are ignored.  No workspace.
 */
rkv_status rkv_compact_inplace(const rkv_params* prm, void* k, void* v, const int32_t* kept_idx, void* stream);

/*
 * The whole step (Sec. 3.1-3.4, Alg. 1): the four calls above back to back on `stream`
 * without host synchronisation.  kept_idx [P, H, budget] and score [P, H, n] are optional
 * outputs (NULL to skip).  Returns RKV_NOT_TRIGGERED without enqueuing anything when
 * N <= budget.  With lambda == 1 the score of Eq. 7 is the importance alone (attention-only
 * eviction, the baseline of Sec. 4) and the similarity pass is skipped.
 */
rkv_status rkv_compress(const rkv_params* prm, const void* q_obs, const void* k, const void* v,
                        void* k_out, void* v_out, int32_t* kept_idx, float* score,
                        void* ws, size_t ws_bytes, void* stream);

/*
 * rkv_compress with the compaction of rkv_compact_inplace as its last stage: k and v are both the
 * input cache [P, H, N, d] and, in their first `budget` rows, the output.  Same optional outputs,
 * statuses and workspace as rkv_compress.
 */
rkv_status rkv_compress_inplace(const rkv_params* prm, const void* q_obs, void* k, void* v, int32_t* kept_idx,
                                float* score, void* ws, size_t ws_bytes, void* stream);

/*
 * rkv_compress for callers that cannot allocate device memory or pass a workspace: code running under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without ws),
 * same kernels, same results bit for bit and same statuses as rkv_compress; the scratch is a fixed array of
 * RKV_STATIC_SCRATCH_BYTES that the library holds on every GPU it runs on until the process ends.  The call
 * allocates and frees nothing, sets no memory with a runtime call and does not synchronise; the first call
 * on each GPU looks the array's address up once (make that call before a capture starts).
 *   - Shapes whose rkv_workspace_size() exceeds RKV_STATIC_SCRATCH_BYTES return RKV_ERR_WORKSPACE with
 *     nothing enqueued (the limit covers one sequence of the 8B model at budget 1024: 32 layers x 8 heads,
 *     N = 1152, about 18 MiB).
 *   - All calls on one GPU share that GPU's array, whatever their stream: calls that overlap in time on one
 *     GPU race and give unspecified results.  Calls on one stream, or ordered by events, are safe; the
 *     array needs no clearing between calls.
 */
#define RKV_STATIC_SCRATCH_BYTES (32u << 20)
rkv_status rkv_compress_static(const rkv_params* prm, const void* q_obs, const void* k, const void* v,
                               void* k_out, void* v_out, int32_t* kept_idx, float* score, void* stream);

/*
 * Instrumented form of rkv_compress for measurement: identical work, and additionally records the
 * five caller-created hipEvent_t handles events[0..4] (a HOST array) on `stream` before the key
 * pre-pass and after the pre-pass, the similarity pass, the finalize/select kernel and the gather,
 * so that hipEventElapsedTime(events[i], events[i+1]) is the duration of stage i.
 */
rkv_status rkv_compress_events(const rkv_params* prm, const void* q_obs, const void* k, const void* v,
                               void* k_out, void* v_out, int32_t* kept_idx, float* score,
                               void* ws, size_t ws_bytes, void* stream, void* const* events);

/*
 * Measurement aid, not a step of the method: one launch that issues nothing but the bf16 MFMA instruction
 * the similarity pass (Eq. 5) is built from, in chains of eight on fragments cut from the caller's data, on
 * every SIMD of the device (two workgroups of four waves per compute unit).  Timed over a few dozen
 * back-to-back launches it gives the rate the matrix pipe SUSTAINS on such data at the clock the chip
 * settles at, which is what the similarity kernel's rate is to be read against (the published peak assumes
 * the top clock).
 *   operands  device, 16-byte aligned, RKV_PROBE_OPERAND_BYTES of bf16 values (e.g. the start of a key
 *             cache); read only
 *   sink      device, RKV_PROBE_SINK_BYTES, overwritten (one float per thread; content of no interest)
 *   chains    chains of eight MFMAs per wave, 1 .. 2^20
 *   flops     host pointer or NULL: receives the floating-point operations of the launch
 * Asynchronous on `stream`.  RKV_ERR_NULL / RKV_ERR_PARAM / RKV_ERR_SHAPE (alignment) before anything is
 * enqueued, RKV_ERR_WORKSPACE if the device has more compute units than the sink is sized for.
 */
#define RKV_PROBE_OPERAND_BYTES (64u << 10)
#define RKV_PROBE_SINK_BYTES (1u << 20)
rkv_status rkv_probe_mfma(const void* operands, void* sink, int chains, void* stream, int64_t* flops);

/*
 * Decode-loop bookkeeping (Sec. 3.1; query cache of App. C.1).  The cache holds up to
 * N = n_tokens = B_budget + B_buffer rows per head; a decode step appends one row.
 *
 * rkv_should_compress: host-only trigger test of Alg. 1.  Returns RKV_OK when `cached_tokens` rows
 * are held and the buffer is full (cached_tokens >= N > budget), RKV_NOT_TRIGGERED otherwise.
 *
 * rkv_cache_append: writes the new token's key/value rows k_new, v_new [P, kv_heads, d] at row
 * `position` (0 <= position < N) of k_cache, v_cache [P, kv_heads, N, d] (strides from rkv_params)
 * and its query state q_new [P, q_heads, d] into slot `q_slot` (0 <= q_slot < alpha) of the query
 * cache q_cache [P, q_heads, alpha, d], which is what rkv_compress takes as q_obs (the importance
 * score does not depend on the order of the alpha slots).  All bf16, device pointers.
 */
rkv_status rkv_should_compress(const rkv_params* prm, int32_t cached_tokens);
rkv_status rkv_cache_append(const rkv_params* prm, void* k_cache, void* v_cache, void* q_cache,
                            const void* k_new, const void* v_new, const void* q_new,
                            int32_t position, int32_t q_slot, void* stream);

/* Static, NUL-terminated description of a status value. */
const char* rkv_status_string(rkv_status s);

#ifdef __cplusplus
}
#endif
#endif /* RKV_H */
