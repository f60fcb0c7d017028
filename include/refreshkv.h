/*
 * refreshkv.h -- C ABI of the RefreshKV decode-attention library for AMD MI355X (gfx950).
 *
 * RefreshKV (arXiv 2411.05787, Section 2.2 "Methodology and Implementation") decodes with
 * two KV caches per layer: the full cache C_f, which is never evicted, and a small cache
 * C_p of K rows that is rebuilt from C_f after every full-attention step.  This library
 * holds the attention-side hot path of one layer:
 *
 *   rk_full_attn        full-attention step over C_f that also returns the attention
 *                       scores of the current token            (Section 2.2, "Decoding with
 *                       full cache"; Appendix A.1 "Compatibility with Flash Attention")
 *   rk_topk_select      the K tokens that refresh C_p: max over the query heads of a GQA
 *                       group, max-pool over neighbouring tokens, top-K
 *                       (Section 2.2 "Prefilling stage" + its GQA footnote; Appendix A.1
 *                       "Baseline Settings": kernel size 7; Appendix A.3)
 *   rk_full_attn_select the two steps above in one call (what a full step of the method does)
 *   rk_score_select     scores over C_f and the selection without the attention output
 *                       (Section 4.3, the "w/o full attention" setting)
 *   rk_window_select    the selection from the scores of the last W prompt tokens: how C_p
 *                       starts after the prefill (Section 2.2 "Prefilling stage"; Appendix A.1)
 *   rk_gather_small_kv  rebuild C_p from the selected rows of C_f         (Section 2.2)
 *   rk_partial_attn     partial-attention step over C_p plus the tokens decoded since the
 *                       refresh                      (Section 2.2, "Decoding with partial cache")
 *   rk_query_sim        the query-similarity test that decides whether a full step is
 *                       needed          (Section 2.2, "Deciding when to decode with full cache")
 *
 * General rules
 * -------------
 * - Every tensor pointer is a DEVICE pointer owned by the caller; `stream` is a hipStream_t
 *   passed as void* (NULL = the default stream).  A call validates its arguments on the host,
 *   then only enqueues kernels on `stream`: it never synchronises, allocates or frees, and the
 *   library keeps no state between calls.  Calls that share a workspace must be ordered on one
 *   stream (or otherwise serialised).
 * - bf16 tensors are 16-bit patterns (upper half of IEEE fp32).  head_dim must be 128, rows of
 *   128 elements are contiguous, and K/V base pointers and strides must keep rows 16-byte
 *   aligned.  q must be 16-byte aligned; out needs 2-byte alignment only, but 8-byte alignment
 *   (any freshly allocated tensor, any [.., n_q_heads, 128] slice of one) lets a row leave in
 *   8-byte stores.  Strides are counted in elements.
 * - Query head h reads KV head h / G with G = n_q_heads / n_kv_heads (1 <= G <= 8).
 * - `seq_lens` is a device int32[batch]: the number of valid rows of each sequence in C_f, the
 *   current token included.  `max_len` is a host-side upper bound of it, used to size grids; a
 *   sequence longer than `max_len` is processed only up to `max_len`.
 * - `pred` / `pred_val`: optional device int32[batch] predicate.  When `pred` is not NULL the
 *   call does nothing for sequence b unless pred[b] == pred_val.  This lets a caller enqueue
 *   both branches of the dynamic schedule without reading the trigger back to the host.
 * - Return value: RK_OK, or a negative rk_status.  On error nothing was enqueued.
 *   Arithmetic: bf16 inputs, fp32 accumulation, bf16 outputs (round to nearest even).
 */
#ifndef REFRESHKV_H
#define REFRESHKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum rk_status {
    RK_OK = 0,
    RK_ERR_INVALID_ARG = -1,   /* NULL pointer, non-positive size, misaligned pointer/stride  */
    RK_ERR_UNSUPPORTED = -2,   /* head_dim != 128, G > 8, k too large, unknown aggregation ... */
    RK_ERR_WORKSPACE   = -3,   /* workspace NULL, misaligned or smaller than rk_workspace_bytes */
    RK_ERR_HIP         = -4,   /* a HIP runtime call failed (launch error)                    */
    RK_ERR_STATIC_SCRATCH = -5 /* the call needs more scratch than the library's built-in array
                                  holds (rk_partial_attn_static); nothing was enqueued            */
} rk_status;

#define RK_AGG_MAX 0           /* aggregation across the query heads of a GQA group: max      */
#define RK_AGG_MEAN 1          /* ... mean (heads added in order in fp32, then divided by G)  */
#define RK_AGG_FIRST 2         /* ... the score of the group's first head (Appendix A.3)      */

#define RK_HEAD_DIM 128
#define RK_MAX_GROUP 8
#define RK_MAX_K 16384         /* largest small-cache size rk_topk_select accepts              */
#define RK_MAX_POOL_W 63       /* largest (odd) max-pool window                                */
#define RK_MAX_SELECT_LEN (1 << 28) /* longest row (max_len) the selection entry points accept  */
#define RK_MAX_WINDOW 32       /* largest observation window rk_window_select accepts          */

/* Geometry of one attention layer; `scale` multiplies q.k before the softmax. */
typedef struct rk_geom {
    int32_t batch;
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    float   scale;
} rk_geom;

/* A KV cache: k and v are bf16 [batch, n_kv_heads, capacity, head_dim] with element strides
 * stride_b (between sequences) and stride_h (between KV heads); the row stride is head_dim.
 * `capacity` is the number of rows allocated per (sequence, KV head): the kernels never touch
 * a row at or beyond it, whatever the device-side lengths and indices say.  Strides are
 * non-negative multiples of 8 elements; stride_h must be below 2^31 (RK_ERR_UNSUPPORTED). */
typedef struct rk_kv {
    const void* k;
    const void* v;
    int64_t stride_b;
    int64_t stride_h;
    int64_t capacity;
} rk_kv;

/* Library version (major * 10000 + minor * 100 + patch). */
int rk_version(void);

/* Static string for a status code. */
const char* rk_status_string(int status);

/* Bytes of device workspace that any call of this library needs for the given geometry, a
 * context of at most max_len rows and a small cache of at most max_k rows.  Host-only. */
size_t rk_workspace_bytes(const rk_geom* geom, int32_t max_len, int32_t max_k);

/* Prepare a workspace (256-byte aligned device memory of at least rk_workspace_bytes) for its
 * first use with this geometry: clears all workspace_bytes of it (a fill kernel on `stream`; no
 * memset, so the call may sit in a captured graph).  The kernels keep arrival counters, call
 * numbers and the tags of partial results there, which must start at zero.  Call once after
 * allocating it, on the stream that will use it; the kernels leave it fit for the next call, so
 * no further initialisation is needed.  A workspace belongs to one geometry (batch and head
 * counts): initialise it again before using it with another. */
int rk_workspace_init(const rk_geom* geom, void* workspace, size_t workspace_bytes, void* stream);

/* Full-attention decode step.
 *   for every sequence b and query head h (KV head g = h / G), over rows j < seq_lens[b]:
 *     s[j]   = scale * <q[b,h,:], K[b,g,j,:]>
 *     a[j]   = exp(s[j] - max_j s) / sum_j exp(s[j] - max_j s)
 *     out[b,h,:] = sum_j a[j] * V[b,g,j,:]              lse[b,h] = log sum_j exp(s[j])
 *   q       bf16 [batch, n_q_heads, 128] contiguous
 *   full    the cache C_f
 *   out     bf16 [batch, n_q_heads, 128] contiguous
 *   weights fp32 [batch, n_q_heads, w_stride] or NULL: weights[b,h,j] = a[j] for
 *           j < seq_lens[b]; other entries are not written.  w_stride >= max_len.  A 16-byte
 *           aligned pointer and a w_stride that is a multiple of 4 let the scores leave in 16-byte
 *           stores (otherwise 4-byte stores: the call is about 10% slower).
 *   lse     fp32 [batch, n_q_heads] or NULL.
 * A sequence with seq_lens[b] == 0 gets out = 0 and lse = -inf. */
int rk_full_attn(const rk_geom* geom, const void* q, rk_kv full,
                 const int32_t* seq_lens, int32_t max_len,
                 void* out, float* weights, int64_t w_stride, float* lse,
                 const int32_t* pred, int32_t pred_val,
                 void* workspace, size_t workspace_bytes, void* stream);

/* First phase of rk_full_attn by itself: the kernel that streams C_f once.  It writes the raw
 * scores scores[b,h,j] = scale * <q[b,h,:], K[b,g,j,:]> (j < seq_lens[b]) and leaves per-chunk
 * partial results in the workspace; out, lse and the normalised weights are NOT produced
 * (rk_full_attn = this kernel + a short finishing kernel that merges the partial results and
 * turns the scores into weights; Section 2.2 "Decoding with full cache", Appendix A.1).
 * Exposed so that a benchmark can time the HBM-bound kernel alone, launch after launch.
 * scores: fp32 [batch, n_q_heads, s_stride], s_stride >= max_len; or NULL: the raw scores stay in the
 * workspace, arranged as the full steps of rk_full_attn_select, rk_full_attn_pool and
 * rk_full_attn_deferred keep them (for groups of 4 query heads: the 4 scores of a position side by
 * side), i.e. the launch is exactly the first kernel of those steps. */
int rk_full_attn_scores(const rk_geom* geom, const void* q, rk_kv full,
                        const int32_t* seq_lens, int32_t max_len,
                        float* scores, int64_t s_stride,
                        const int32_t* pred, int32_t pred_val,
                        void* workspace, size_t workspace_bytes, void* stream);

/* Selection of the rows that refresh the small cache.
 *   for every sequence b and KV head g, with n = seq_lens[b]:
 *     A[j] = max over the G heads h of group g of weights[b,h,j]
 *     P[j] = max of A over the window of pool_w positions centred on j, clipped to [0, n)
 *     idx[b,g,0 .. k') = the k' = min(k, n) positions of largest P, ordered by P descending,
 *                        equal P by ascending position;  idx[b,g,k' .. k) = -1
 *     sel_scores[b,g,i] = P[idx[b,g,i]] (0 where idx is -1), when sel_scores is not NULL
 *   weights must be non-negative and free of NaN (softmax output).  pool_w odd, 1..63
 *   (7 in the paper, 1 = no pooling).  agg: RK_AGG_MAX (the method's choice; then A is the max
 *   above), RK_AGG_MEAN or RK_AGG_FIRST (the alternatives of Appendix A.3).  1 <= k <= RK_MAX_K.
 *   max_len <= RK_MAX_SELECT_LEN (RK_ERR_UNSUPPORTED beyond; the same limit holds for every entry
 *   point that selects).
 *   idx int32 [batch, n_kv_heads, k]; sel_scores fp32 of the same shape or NULL. */
int rk_topk_select(const rk_geom* geom, const float* weights, int64_t w_stride,
                   const int32_t* seq_lens, int32_t max_len,
                   int32_t k, int32_t pool_w, int32_t agg,
                   int32_t* idx, float* sel_scores,
                   const int32_t* pred, int32_t pred_val,
                   void* workspace, size_t workspace_bytes, void* stream);

/* The two calls above in one: a full-attention step whose attention weights go straight into
 * the selection (Section 2.2, "Decoding with full cache": every full step is followed by the
 * refresh of the small cache).  Results are those of rk_full_attn followed by rk_topk_select on
 * its weights; the weights stay in the workspace between the kernels, one launch and one pass
 * over them are saved.  `weights` may be NULL when the caller does not want them returned
 * (otherwise as in rk_full_attn); every other argument as in the two calls. */
int rk_full_attn_select(const rk_geom* geom, const void* q, rk_kv full,
                        const int32_t* seq_lens, int32_t max_len,
                        void* out, float* weights, int64_t w_stride, float* lse,
                        int32_t k, int32_t pool_w, int32_t agg,
                        int32_t* idx, float* sel_scores,
                        const int32_t* pred, int32_t pred_val,
                        void* workspace, size_t workspace_bytes, void* stream);

/* rk_full_attn_select in two halves, for callers that overlap the selection with other work.
 * The step's output is complete after the first half; the selection and the gather are needed
 * only by the NEXT partial step of the same layer, so they can run on another stream beside the
 * attention of the following layers.
 *   rk_full_attn_pool   everything of rk_full_attn_select up to and including the pooled group
 *                       scores and their histogram, which stay in `workspace`;
 *   rk_select_pooled    the top-K from what rk_full_attn_pool left in the SAME workspace, with the
 *                       same seq_lens, max_len, predicate and geometry.
 * beside_other_work != 0: the attention kernel is launched in more, smaller workgroups (two
 * residency waves): 5-10% slower when it has the GPU to itself, but kernels of another stream (the
 * selections and gathers of earlier layers) can start while it runs; 0: the launch shape of
 * rk_full_attn_select.
 * Between the two calls no other call may use that workspace (two workspaces used in turn let the
 * next layer's rk_full_attn_pool start before this layer's rk_select_pooled has run).  The pair
 * leaves the workspace as clean as rk_full_attn_select does. */
int rk_full_attn_pool(const rk_geom* geom, const void* q, rk_kv full,
                      const int32_t* seq_lens, int32_t max_len,
                      void* out, float* weights, int64_t w_stride, float* lse,
                      int32_t pool_w, int32_t agg, int32_t beside_other_work,
                      const int32_t* pred, int32_t pred_val,
                      void* workspace, size_t workspace_bytes, void* stream);
int rk_select_pooled(const rk_geom* geom, const int32_t* seq_lens, int32_t max_len, int32_t k,
                     int32_t* idx, float* sel_scores, const int32_t* pred, int32_t pred_val,
                     void* workspace, size_t workspace_bytes, void* stream);

/* Scores-only refresh (Section 4.3 "Impact of full attention steps", the setting "w/o full
 * attention": the attention scores over the entire cache are calculated and the small cache is
 * updated from them; the step's output then comes from rk_partial_attn on the updated small
 * cache, so the values of the full cache are never read: half the bytes of a full step).
 * Computes weights[b,h,j] = softmax_j(scale * <q[b,h,:], K[b,g,j,:]>), j < seq_lens[b], and the
 * selection of rk_topk_select on them, exactly as rk_full_attn_select does, but produces no
 * attention output.  full.v is not read and may be NULL.  `weights` ([batch, n_q_heads,
 * w_stride] fp32) and `lse` are optional outputs (NULL: not returned); the other arguments as in
 * rk_full_attn_select. */
int rk_score_select(const rk_geom* geom, const void* q, rk_kv full,
                    const int32_t* seq_lens, int32_t max_len,
                    float* weights, int64_t w_stride, float* lse,
                    int32_t k, int32_t pool_w, int32_t agg,
                    int32_t* idx, float* sel_scores,
                    const int32_t* pred, int32_t pred_val,
                    void* workspace, size_t workspace_bytes, void* stream);

/* Prefill-side initialisation of the small cache from an observation window (Section 2.2
 * "Prefilling stage": the small cache starts from the attention scores of the last prompt token;
 * Section 3 describes the SnapKV baseline as the tokens with high scores from the last few tokens
 * of the prompt, and Appendix A.1 "Baseline Settings" calls their number the observation window
 * size: 1 in the paper's runs, where this call selects what rk_score_select selects).
 *   q_win   bf16 [batch, window, n_q_heads, 128]: entry i is the query of the prompt token at
 *           position p_i = seq_lens[b] - window + i, so the last entry belongs to the last prompt
 *           token.  Entries with p_i < 0 (prompt shorter than the window) are ignored.
 *   full    the full cache with the whole prompt appended; only full.k is read (full.v may be NULL)
 *   votes[b,h,j] = sum_i softmax_{j' <= p_i}(scale * <q_win[b,i,h,:], K[b,g,j',:]>)[j]   (causal:
 *           query i sees rows 0..p_i), the rule of the cited work for a window of several queries.
 *           Optional output, fp32 [batch, n_q_heads, v_stride], v_stride >= max_len; positions
 *           >= seq_lens[b] are not written.  NULL: kept in the workspace only.
 *   idx, sel_scores, k, pool_w, agg: the selection of rk_topk_select applied to the votes; all
 *           rows of the prompt compete, the window's own rows included.
 *   1 <= window <= RK_MAX_WINDOW (RK_ERR_UNSUPPORTED beyond).  The other arguments as in
 *   rk_score_select.  K is read twice (log-sum-exp of every query first, votes second). */
int rk_window_select(const rk_geom* geom, const void* q_win, int32_t window, rk_kv full,
                     const int32_t* seq_lens, int32_t max_len,
                     float* votes, int64_t v_stride,
                     int32_t k, int32_t pool_w, int32_t agg,
                     int32_t* idx, float* sel_scores,
                     const int32_t* pred, int32_t pred_val,
                     void* workspace, size_t workspace_bytes, void* stream);

/* Rebuild the small cache: small.k[b,g,i,:] = full.k[b,g,idx[b,g,i],:] and the same for v, for
 * every i < k with idx >= 0 (bit copies).  Slots whose idx is negative are left untouched.
 * A slot whose idx is >= the capacity of `full` is skipped as well.  `small` must hold at least
 * k rows per head and is written through its (const-declared) pointers.
 * Refresh bookkeeping in the same launch: when tail_start is not NULL (seq_lens then required),
 * tail_start[b] = seq_lens[b] for every sequence the predicate selects, i.e. the rows "decoded
 * since the refresh" start at the current length (what rk_mark_refresh does on its own). */
int rk_gather_small_kv(const rk_geom* geom, rk_kv full, const int32_t* idx, int32_t k,
                       rk_kv small, const int32_t* seq_lens, int32_t* tail_start,
                       const int32_t* pred, int32_t pred_val, void* stream);

/* Partial-attention decode step: the softmax attention of rk_full_attn, but over the row list
 *   small rows 0 .. min(n_sel, tail_start[b]) - 1, then
 *   full  rows tail_start[b] .. seq_lens[b] - 1   (the tokens decoded since the refresh,
 *                                                  the current one included)
 * tail_start is a device int32[batch]: seq_lens at the last refresh.  max_recent is a host
 * upper bound of seq_lens[b] - tail_start[b].  With n_sel = K all selected rows are read;
 * with n_sel = K - (seq_lens - tail_start) the small cache keeps a fixed size and drops its
 * lowest-scored rows first (the small cache is in descending score order).
 * No attention scores are returned.  An empty row list gives out = 0. */
int rk_partial_attn(const rk_geom* geom, const void* q, rk_kv small, int32_t n_sel,
                    rk_kv full, const int32_t* tail_start, const int32_t* seq_lens,
                    int32_t max_recent, void* out,
                    const int32_t* pred, int32_t pred_val,
                    void* workspace, size_t workspace_bytes, void* stream);

/* rk_partial_attn for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments less the
 * workspace, same kernels, same results bit for bit.  The step's scratch (arrival counters,
 * per-workgroup softmax statistics and partial outputs) is a device array built into the library,
 * RK_STATIC_SCRATCH_BYTES per GPU, held from the moment the library is loaded until the process
 * ends; the call allocates and frees nothing and calls no library that does.
 * Limits: batch * n_kv_heads <= 4096 and rk_partial_attn_static_bytes(geom, n_sel, max_recent) <=
 * RK_STATIC_SCRATCH_BYTES (any step of up to 256 (sequence, KV head) pairs fits, whatever its
 * n_sel, max_recent and group size); beyond them the call returns RK_ERR_STATIC_SCRATCH and
 * enqueues nothing.  The device that is current when the call is made must be the stream's.  On
 * its first call on a device the library looks the array up on that device and enqueues one small
 * fill kernel ahead of the step.  All calls on one GPU share that GPU's array: calls that may
 * overlap in time (different streams without an ordering between them, several host threads whose
 * streams run concurrently) race on it and must be serialised by the caller. */
#define RK_STATIC_SCRATCH_BYTES (8u << 20)
size_t rk_partial_attn_static_bytes(const rk_geom* geom, int32_t n_sel, int32_t max_recent);
int rk_partial_attn_static(const rk_geom* geom, const void* q, rk_kv small, int32_t n_sel,
                           rk_kv full, const int32_t* tail_start, const int32_t* seq_lens,
                           int32_t max_recent, void* out,
                           const int32_t* pred, int32_t pred_val, void* stream);

/* The same step with the fixed-size small cache of Section 2.2 ("Decoding with partial cache":
 * the new token's KV pair is appended to C_p and the KV pair with the lowest score is evicted):
 * sequence b reads the first max(k - r[b], 0) selected rows, r[b] = seq_lens[b] - tail_start[b]
 * being the rows decoded since its refresh, plus those r[b] rows from the full cache, so k rows
 * in all.  Equal to rk_partial_attn with n_sel = k - r when every sequence has the same r; here
 * r is taken per sequence on the GPU (dynamic schedule, ragged batches). */
int rk_partial_attn_fixed(const rk_geom* geom, const void* q, rk_kv small, int32_t k,
                          rk_kv full, const int32_t* tail_start, const int32_t* seq_lens,
                          int32_t max_recent, void* out,
                          const int32_t* pred, int32_t pred_val,
                          void* workspace, size_t workspace_bytes, void* stream);

/* The first partial step after a refresh whose rk_gather_small_kv was left out (the gather moved
 * into the step that first needs its result: Section 2.2's small cache is still rebuilt, by the
 * kernel that reads it).  Computes what rk_partial_attn (fixed_size = 0, n_sel = k) or
 * rk_partial_attn_fixed (fixed_size = 1) computes on a small cache rebuilt from `idx`, but takes the
 * selected rows from the full cache through idx (int32 [batch, n_kv_heads, k], as rk_topk_select
 * leaves it) and writes them into `small` on the way: afterwards, for every selected row i the step
 * attended to, small.k[b,g,i,:] = full.k[b,g,idx[b,g,i],:] and the same for v, bit for bit (with
 * fixed_size = 0 these are all min(k, tail_start[b]) rows; with fixed_size = 1 the rows the step no
 * longer reads are not written, and no later step reads them either).  Later partial steps use
 * rk_partial_attn / rk_partial_attn_fixed on `small` as usual.  tail_start must already hold the
 * refresh's value (rk_mark_refresh).  An idx entry outside [0, full.capacity) is clamped into the
 * cache (none occurs among the entries rk_topk_select writes for existing rows).  k >= 1 and
 * small.capacity >= k; the other arguments as in rk_partial_attn. */
int rk_partial_attn_lazy(const rk_geom* geom, const void* q, rk_kv small, const int32_t* idx, int32_t k,
                         int32_t fixed_size, rk_kv full, const int32_t* tail_start, const int32_t* seq_lens,
                         int32_t max_recent, void* out,
                         const int32_t* pred, int32_t pred_val,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Query-similarity trigger.
 *   qbar[b,:] = mean over the query heads of q[b,h,:]                        (fp32)
 *   sim[b]    = <qbar, q_ref[b]> / (max(|qbar|, 1e-8) * max(|q_ref[b]|, 1e-8))
 *   need_full[b] = (sim[b] <= threshold) || force_full
 *   if need_full[b]: q_ref[b,:] = qbar[b,:]
 * q_ref fp32 [batch, 128] is read and updated in place (16-byte aligned, like q:
 * RK_ERR_INVALID_ARG otherwise); sim fp32 [batch]; need_full int32 [batch] (0/1).  The sums are
 * taken in fp32 in a fixed order (so every call gives the same bits for the same input).  Pass force_full = 1 on steps that are full by schedule (fixed stride,
 * first step) so that the reference follows the most recent full step. */
int rk_query_sim(const rk_geom* geom, const void* q, float* q_ref, float threshold,
                 int32_t force_full, float* sim, int32_t* need_full, void* stream);

/* The trigger's test and the partial step it guards in one launch (Section 2.2, "Deciding when
 * to decode with full cache": the similarity check is to cost as little as possible).  For every
 * sequence b, with sim and the decision as in rk_query_sim with force_full = 0:
 *   sim[b], need_full[b] are stored;
 *   need_full[b] == 0: out[b] as rk_partial_attn (fixed_size == 0, n_sel rows of `small`) or
 *                      rk_partial_attn_fixed (fixed_size != 0, k = n_sel) leaves it; q_ref[b] unchanged;
 *   need_full[b] == 1: out[b] is not written, q_ref[b,:] = qbar[b,:]; the caller's full step follows
 *                      under the predicate (need_full, 1).
 * The same result as rk_query_sim followed by the partial step under the predicate (need_full, 0),
 * without the launch of the test and without the partial step waiting for it: every workgroup of
 * the step works the test out for itself while its first rows are on their way.  Arguments as in
 * rk_query_sim and rk_partial_attn; q_ref, sim and need_full must not be NULL. */
int rk_partial_attn_triggered(const rk_geom* geom, const void* q, rk_kv small, int32_t n_sel,
                              int32_t fixed_size, rk_kv full, const int32_t* tail_start,
                              const int32_t* seq_lens, int32_t max_recent, void* out,
                              float* q_ref, float threshold, float* sim, int32_t* need_full,
                              void* workspace, size_t workspace_bytes, void* stream);

/* Plain device-to-device copy of `bytes` bytes (a multiple of 16; both pointers 16-byte aligned)
 * with 16-byte loads and stores, one launch.  It exists so that a profiler run of the benchmark
 * holds a kernel whose HBM traffic is known exactly (bytes read + bytes written), against which
 * the byte counters read for the attention kernels are scaled. */
int rk_calibration_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Reads `bytes` bytes (a multiple of 16; src 16-byte aligned) with 16-byte streaming loads and
 * keeps nothing (sink: one device word that is written only if the words read xor to one fixed
 * value).  It exists so that the benchmark can report, beside the attention kernels, the rate a
 * kernel that only reads reaches on the same GPU. */
int rk_calibration_read(const void* src, size_t bytes, uint32_t* sink, void* stream);

/* Test hook.  In launches small enough for all their workgroups to run at once, the partial step and
 * rk_full_attn without weights let every workgroup merge a share of the output, each re-reading the
 * other workgroups' partial results while these are still on their way.  `spin` (>= 0; default 256) bounds
 * those re-reads: a workgroup that exceeds it leaves its share to the workgroup that publishes last, which
 * waits for nobody.  0 makes every workgroup hand over at once, so that a test can drive that path; results
 * are the same bits for any value.  Process-wide, read when a call is enqueued.  Returns RK_ERR_INVALID_ARG
 * for a negative value. */
int rk_debug_set_slice_spin(int32_t spin);

/* Bookkeeping of a refresh: tail_start[b] = seq_lens[b] for every sequence the predicate
 * selects (all when pred is NULL).  After a full step + refresh the rows "decoded since the
 * refresh" start at the current length (Section 2.2: the partial cache then grows by the
 * tokens decoded with it).  Both arrays are device int32[batch]. */
int rk_mark_refresh(const rk_geom* geom, const int32_t* seq_lens, int32_t* tail_start,
                    const int32_t* pred, int32_t pred_val, void* stream);

/* ---- the H2O comparison policy on the same attention step --------------------------------- */

/* H2O (Section 3 "Comparison systems": the recent tokens plus dynamically updated "heavy hitters",
 * the tokens with high cumulative attention scores; Appendix A.1 "Baseline Settings": K/2 each, the
 * scores aggregated over a GQA group by max as for the paper's own method; Section 4.1: it needs
 * the attention scores at every decoding step, which is what makes it slow).  Per (sequence, KV
 * head) and step: the new token joins the cache; the step attends over the whole cache and every
 * cached token adds the aggregated score it received to its running total (fp32); if the cache
 * then holds more than `budget` tokens, the one with the lowest total among those whose position
 * is <= newest - recent is dropped for good (equal totals: the older one).
 * State, all caller-owned device memory.  Slots are dense ([0, n_rows)) but not in token order:
 * the newest token moves into the slot of the dropped one. */
typedef struct rk_h2o_state {
    rk_kv cache;           /* rows of the kept tokens; capacity >= budget + 1                   */
    float* total;          /* fp32 [batch, n_kv_heads, cache.capacity]: running totals          */
    int32_t* pos;          /* int32 [batch, n_kv_heads, cache.capacity]: token position per slot */
    int32_t* n_rows;       /* int32 [batch]: tokens kept (the same for every head)              */
    int32_t* n_attend;     /* int32 [batch]: rows the current step attends over (written by
                              rk_h2o_append, read by the attention and by rk_h2o_update)        */
} rk_h2o_state;

/* The three parts of a step; rk_h2o_step enqueues all of them.
 *   rk_h2o_append  rows k_new, v_new (bf16 [batch, n_kv_heads, 128]) go to slot n_rows[b] with
 *                  total 0 and position seq_lens[b] - 1 (seq_lens: tokens so far, the new one
 *                  included); n_attend[b] = n_rows[b] + 1.
 *   (attention)    rk_full_attn over state.cache with seq_lens = state.n_attend, max_len =
 *                  budget + 1 and `weights` returned.
 *   rk_h2o_update  totals += aggregate over the group of weights[b,h,j] ([batch, n_q_heads,
 *                  w_stride] fp32, w_stride >= budget + 1), drop rule, n_rows[b] updated;
 *                  dropped (optional, int32 [batch, n_kv_heads]) gets the position dropped or -1.
 *   rk_h2o_step    the three in one call; the scores pass through `workspace`
 *                  (rk_workspace_bytes(geom, budget + 1, 0) or more).  out bf16 [batch,
 *                  n_q_heads, 128].
 * 0 <= recent < budget; agg as in rk_topk_select. */
int rk_h2o_append(const rk_geom* geom, rk_h2o_state state, const void* k_new, const void* v_new,
                  const int32_t* seq_lens, int32_t budget, void* stream);
int rk_h2o_update(const rk_geom* geom, rk_h2o_state state, const float* weights, int64_t w_stride,
                  int32_t budget, int32_t recent, int32_t agg, int32_t* dropped, void* stream);
int rk_h2o_step(const rk_geom* geom, rk_h2o_state state, const void* q,
                const void* k_new, const void* v_new, const int32_t* seq_lens,
                int32_t budget, int32_t recent, int32_t agg,
                void* out, int32_t* dropped,
                void* workspace, size_t workspace_bytes, void* stream);

/* ---- one decode step of a whole model --------------------------------------------------- */

/* Per-layer state of the method: everything is caller-owned device memory. */
typedef struct rk_layer_state {
    rk_kv full;            /* C_f of the layer                                                  */
    rk_kv small;           /* C_p of the layer, capacity >= k                                   */
    int32_t* idx;          /* int32 [batch, n_kv_heads, k]: the selection of the last refresh   */
    int32_t* tail_start;   /* int32 [batch]: seq_lens at the last refresh                       */
    float* q_ref;          /* fp32 [batch, head_dim]: reference query of the trigger (dynamic)  */
    float* sim;            /* fp32 [batch]: last similarity (dynamic)                           */
    int32_t* need_full;    /* int32 [batch]: last decision of the trigger (dynamic)             */
    int32_t* n_full;       /* int32 [batch] or NULL: incremented at every refresh of (layer,
                              sequence): step count / n_full is the effective stride of App.
                              "Effective stride per layer"                                      */
} rk_layer_state;

/* The schedule of Section 2.2 and the two variants of the step. */
typedef struct rk_schedule {
    int32_t k;             /* small-cache size K                                                */
    int32_t pool_w;        /* max-pool window of the selection (7 in the paper)                 */
    int32_t stride;        /* S (fixed schedule) or the QC stride (dynamic); <= 0: never after
                              the initialisation                                                */
    int32_t dynamic;       /* 1: the query-similarity trigger decides on every stride-th step   */
    float   threshold;     /* s: full step iff similarity <= s                                  */
    int32_t fixed_size;    /* 1: partial steps use rk_partial_attn_fixed (evict the lowest)     */
    int32_t scores_only;   /* 1: refreshes use rk_score_select + rk_partial_attn (Section 4.3)  */
} rk_schedule;

#define RK_STEP_FULL    1  /* every layer took a full step                                      */
#define RK_STEP_PARTIAL 2  /* every layer took a partial step                                   */
#define RK_STEP_BOTH    3  /* trigger test step: both branches enqueued, predicated per sequence */

/* Attention of decode step t (t = 0: the prefill-equivalent initialisation; steps count from 1)
 * for n_layers layers, enqueued on `stream` in layer order: exactly the calls a caller would
 * issue layer by layer (rk_query_sim, rk_full_attn_select or rk_score_select,
 * rk_gather_small_kv, rk_partial_attn / rk_partial_attn_fixed), with the trigger's device
 * predicate on test steps.  `layers`, `q` and `out` are HOST arrays of n_layers entries
 * (q[l], out[l]: device bf16 [batch, n_q_heads, head_dim]); they are read during the call only.
 * seq_lens (shared by the layers) must already count the current token, whose K/V rows the
 * caller has written to every layer's C_f.  max_len / max_recent: host bounds of seq_lens and
 * of seq_lens - tail_start.  Returns RK_STEP_* (> 0) or a negative rk_status; on an error in
 * layer l the layers before it have been enqueued. */
int rk_decode_step(const rk_geom* geom, const rk_schedule* sched, int32_t t, int32_t n_layers,
                   const rk_layer_state* layers, const void* const* q, void* const* out,
                   const int32_t* seq_lens, int32_t max_len, int32_t max_recent,
                   void* workspace, size_t workspace_bytes, void* stream);

/* What rk_decode_step_overlapped needs besides rk_decode_step's arguments; all caller-owned. */
typedef struct rk_overlap {
    void* side_stream;          /* hipStream_t for the selections and gathers of a full step         */
    void* const* ready;         /* host array of n_layers hipEvent_t: recorded on `stream` when a
                                   layer's pooled scores are complete                              */
    void* const* done;          /* host array of n_layers hipEvent_t: recorded on side_stream when
                                   a layer's small cache is rebuilt                                */
    void* join;                 /* one more hipEvent_t                                             */
    void* const* workspaces;    /* host array of n_workspaces device workspaces of workspace_bytes
                                   each, initialised with rk_workspace_init                        */
    int32_t n_workspaces;       /* >= 2 to overlap (3 measured best); 1: same as rk_decode_step    */
    size_t workspace_bytes;
} rk_overlap;

/* rk_decode_step with the refresh of a full step off the critical path: per layer,
 * rk_full_attn_pool on `stream`, then rk_select_pooled and rk_gather_small_kv on
 * ov->side_stream beside the following layers' full attention; `stream` has waited for all of it
 * when the step's work on it ends.  Same results, same return values.  Other steps, and the
 * scores-only refresh, are passed to rk_decode_step with the first workspace.  The events must
 * not be in use by anything else while the step is in flight.
 * Submit a step that uses the side stream late: if many earlier steps are still pending on
 * `stream`, the side stream's queue sits blocked behind all of them, and on MI355X a blocked queue
 * slows every kernel launch of the other one (about 0.9 us each, measured).  A loop that lets at
 * most one earlier step be pending when it calls this for a full step avoids that. */
int rk_decode_step_overlapped(const rk_geom* geom, const rk_schedule* sched, int32_t t, int32_t n_layers,
                              const rk_layer_state* layers, const void* const* q, void* const* out,
                              const int32_t* seq_lens, int32_t max_len, int32_t max_recent,
                              const rk_overlap* ov, void* stream);

/* Full attention of a full step whose pooling is left for rk_refresh_batched (Section 2.2,
 * "Decoding with full cache"): `out` (and lse, if given) as rk_full_attn; the raw scores of the
 * step and the statistics that normalise them stay in `workspace`, which must not be used for
 * anything else until rk_refresh_batched has run with pool_w != 0.  Launches the same kernels as
 * the first half of rk_full_attn_pool, less the pooling tiles of its finishing kernel. */
int rk_full_attn_deferred(const rk_geom* geom, const void* q, rk_kv full,
                          const int32_t* seq_lens, int32_t max_len, void* out, float* lse,
                          const int32_t* pred, int32_t pred_val,
                          void* workspace, size_t workspace_bytes, void* stream);

/* The refreshes of all layers of a full step at once, after every layer's rk_full_attn_pool
 * (pool_w == 0) or rk_full_attn_deferred (pool_w = the odd pooling width, agg = RK_AGG_*: the
 * scores are pooled here first, all layers in one launch, with the results rk_full_attn_pool
 * would have left): for layer l, rk_select_pooled on workspaces[l] (which holds what that call
 * left for the layer, with the same seq_lens, max_len and geometry) into layers[l].idx, then
 * rk_gather_small_kv into layers[l].small with tail_start <- seq_lens and, where given,
 * n_full += 1.  A layer's selection and gather are needed only by its next partial step (Section
 * 2.2), so they can wait until the last layer's attention is done; here all selections run in one
 * launch and all gathers in another (per 32 layers), which fills the chip where one layer's
 * refresh cannot.  Same results as the per-layer calls.  Every layer needs a workspace of its own
 * (workspace_bytes each); the caches of all layers must share strides and capacity
 * (RK_ERR_UNSUPPORTED otherwise).  by_need_full != 0: layer l refreshes only the sequences with
 * layers[l].need_full[b] == 1 (what the trigger of that layer decided: the scores of the others
 * are stale and are not looked at); 0: every sequence of every layer. */
int rk_refresh_batched(const rk_geom* geom, int32_t n_layers, const rk_layer_state* layers,
                       void* const* workspaces, size_t workspace_bytes,
                       const int32_t* seq_lens, int32_t max_len, int32_t k, int32_t pool_w, int32_t agg,
                       int32_t by_need_full, void* stream);

/* rk_decode_step whose full steps do the refresh with rk_refresh_batched: per layer
 * rk_full_attn_deferred on workspaces[l] (n_layers workspaces of workspace_bytes each, initialised with
 * rk_workspace_init), then one rk_refresh_batched for all layers; on the trigger's test steps both
 * branches are enqueued as in rk_decode_step and the batched refresh goes by every layer's need_full.
 * One stream, no events.  Same results and return values as rk_decode_step; partial steps, and the
 * scores-only refresh, are passed to rk_decode_step with workspaces[0]. */
int rk_decode_step_batched(const rk_geom* geom, const rk_schedule* sched, int32_t t, int32_t n_layers,
                           const rk_layer_state* layers, const void* const* q, void* const* out,
                           const int32_t* seq_lens, int32_t max_len, int32_t max_recent,
                           void* const* workspaces, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* REFRESHKV_H */
