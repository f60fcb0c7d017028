// Shared host-side plumbing of the library: workspace layout, argument checks, launch checks.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/refreshkv.h"

namespace rk {

constexpr int kD = RK_HEAD_DIM;          // head_dim
constexpr int kMinChunk = 128;           // rows one workgroup takes per round: 4 wavefronts x 32
constexpr int kMaxChunks = 256;          // most partial results one (sequence, KV head) produces
constexpr int kMergeChunks = 64;         // ... when the split kernel itself merges them
#ifndef RK_TARGET_WGS
#define RK_TARGET_WGS 768                // workgroups a split launch aims for (3 per CU, all resident)
#endif

// Workgroups per (sequence, KV head) of a split attention launch whose partial results a second
// kernel merges.  Upper bound: as many as give the launch RK_TARGET_WGS workgroups in all (such a
// launch is resident as a whole from the start), never more than `limit` (the most partial
// results the merge takes), never more than there are stretches of kMinChunk rows.
// Below that bound, a count that gives every CU the same number of workgroups is preferred
// (total a multiple of the 256 CUs) as long as no wavefront gets more tiles for it.  Measured on
// the score-emitting kernel alone, 8 KV heads, total workgroups -> us per launch:
//   24576 rows: 512 -> 20.5, 768 -> 21.5, 1024 -> 22.4;   560..720 -> 22.5..25.9
//   32768 rows: 512 -> 27.1, 768 -> 27.5, 1024 -> 26.6;   560..720 -> 28.9..31.6
//   65536 rows: 512 -> 51.5, 768 -> 52.5, 1024 -> 49.7;   560..720 -> 54.5..60.1
// and the same picture with 4 KV heads and with a batch of 4: an even spread is worth 10-20%,
// which of the even spreads is worth 3-5% and depends on the length; 3 per CU (one residency
// wave) is never more than 5% from the best.
// `target` above RK_TARGET_WGS (rk_full_attn_pool: 4 per CU): the launch then runs in two
// residency waves, which costs it 5% when it has the chip to itself (26.7 -> 29.7 us at 32k rows)
// but lets the kernels of a second stream, which do not fit beside three of these workgroups on a
// CU, start while it runs: full step of 32 layers with the refresh on a second stream 46.7 -> 45.3 us
// per layer.
constexpr int kComputeUnits = 256;
constexpr int kCoRunTargetWgs = 1024;
constexpr int kCoRunMaxChunks = 128;     // with 4 KV heads 1024 workgroups are 256 partial results per head: the finish
                                         // then costs more than the co-running gains (46.2 -> 51.5 us per layer)
static inline int split_workgroups(int64_t max_rows, int64_t n_problems, int limit, int target = RK_TARGET_WGS) {
    if (n_problems < 1) n_problems = 1;
    int64_t per = target / n_problems;
    const int64_t stretches = (max_rows + kMinChunk - 1) / kMinChunk;
    if (per > stretches) per = stretches;
    if (per > limit) per = limit;
    if (per < 1) per = 1;
    const int64_t tiles = (max_rows + 31) / 32;
    auto rounds = [&](int64_t nch) { return (tiles + 4 * nch - 1) / (4 * nch); };
    for (int64_t nch = per; nch >= 1 && 8 * nch >= 5 * per; --nch)
        if ((nch * n_problems) % kComputeUnits == 0 && rounds(nch) == rounds(per)) return (int)nch;
    return (int)per;
}

// Workgroups per (sequence, KV head) when the last workgroup of the launch merges the partial
// results inside the kernel (partial steps; short full steps without scores).  There the merge
// sets the terms (measured, K = 1024..8192, groups of 4, 7 and 8): it reads the partial outputs
// in batches of 16 per round trip, and a 17th partial result costs 0.8 us, about what a whole
// further round of tiles costs a wavefront (16 workgroups: 9.1 us, 17: 9.9 at K = 2048; 16: 10.3,
// 33: 13.7 at K = 4096; 16: 14.6, 40: 17.2 at K = 8192).  So: the largest count within whole
// batches of 16 that keeps the rounds per wavefront at 5 or fewer, one batch if possible; and a
// tail of a few rows (the tokens decoded since the refresh) gets no workgroup of its own, one
// wavefront takes it as a second tile.  With several sequences the launch as a whole is best at
// about one workgroup per CU (us per launch by workgroups per (sequence, KV head), 8 KV heads:
// 16 sequences, K = 1024: 1: 21.7, 2: 18.7, 4: 19.5, 6: 20.7, 8: 23.4;  16 x 2048: 2: 28.4, 4: 31.1,
// 6: 33.8, 16: 40.0;  8 x 4096: 2: 33.0, 4: 28.5, 12: 32.1, 32: 45.1;  4 x 2048: 4: 16.5, 8: 13.7,
// 16: 14.1;  64 x 512: 1: 30.1, 2: 33.6), so the upper bound is 256 workgroups in all, not the 768 of
// the kernels that leave the merge to a second launch.
// two_batches: the ticketed merge, which requests two batches of 16 partial outputs before it waits
// for the first: 32 partial results cost it one round trip, so where 16 workgroups would leave every
// wavefront two or more tiles, 32 halve the tiles for nothing (one sequence, 4 KV heads, 7 heads per
// group: K = 4096 10.4 -> 10.0 us, K = 8192 13.8 -> 12.5; 48 and 64 workgroups: 10.3 / 13.0 and more; the
// tagged merge reads 20 partial results per round trip and more rows per result: 32 cost it 16.2
// against 13.0 us at K = 8192, groups of 4).
// (Groups of up to 4 heads: the tagged merge wins while 16 workgroups give a wavefront one tile, the
// ticketed one with 32 workgroups beyond: K = 2048 7.5 / 7.7 us, 4096 9.8 / 9.3, 8192 13.0 / 12.5,
// 16384 23.9 / 18.1; so where this is true and the merge is the last workgroup's, the partial step takes the
// ticketed form whatever the group.  With the merge by slices, below, neither is used for launches over few
// pairs: what is left of this rule serves the workspace without a tagged region.)
static inline bool two_batches_pay(int64_t rows, int64_t tail_rows, int64_t n_problems) {
    const int64_t problems = n_problems > 0 ? n_problems : 1;
    const int64_t main_rows = (rows > 0 && tail_rows <= kMinChunk) ? rows : rows + tail_rows;     // a few rows decoded since the refresh do not count
    return (kComputeUnits + problems / 2) / problems >= 32 && (main_rows + 31) / 32 > 4 * 16;
}
static inline int merged_split_workgroups(int64_t rows, int64_t tail_rows, int64_t n_problems, bool two_batches = false) {
    const int64_t all_rows = rows + tail_rows;
    const int64_t counted = (rows > 0 && tail_rows <= 32) ? rows : all_rows;
    const int64_t problems = n_problems > 0 ? n_problems : 1;
    int64_t per = (kComputeUnits + problems / 2) / problems;        // one workgroup per CU in all, see above
    const int64_t stretches = (counted + kMinChunk - 1) / kMinChunk;
    if (per > stretches) per = stretches;
    if (per > kMergeChunks) per = kMergeChunks;
    if (per < 1) per = 1;
    const int64_t tiles = (all_rows + 31) / 32;
    if (two_batches && two_batches_pay(rows, tail_rows, n_problems)) return 32;
    for (int64_t n = 16; n < per; n += 16)
        if ((tiles + 4 * n - 1) / (4 * n) <= 5) return (int)n;
    return (int)per;
}

// The same for the tagged merge (groups of up to 4 heads) from 16 (sequence, KV head) pairs on; first for 32 and more.
// With many pairs the launch is bound by what a CU gets through, not by one workgroup's chain:
// it takes about (workgroups per CU, rounded up) x (tiles per wavefront + 1 for a workgroup's
// fixed costs), plus a round trip of the merge per 20 partial results beyond the first 20.  A
// total just above a multiple of the 256 CUs is what hurts: the few CUs with one workgroup more set
// the time.  `tail` = 1: the rows decoded since the refresh have a workgroup of their own.
// Measured, us per launch, old rule -> this one (8 KV heads, groups of 4): 16 sequences, K = 1024:
// 22.1 -> 18.9; K = 2048: 37.1 -> 32.3; K = 4096: 68.3 -> 54.1; 8 sequences, K = 1024: 14.6 -> 12.8;
// K = 2048: 23.7 -> 20.6; 4 sequences, K = 2048: 14.4 -> 13.0; K = 8192: 38.2 -> 29.9; 32 x 1024:
// 38.3 -> 33.8 - 35.5; 64 x 512: 39.9 -> 35.0.
// With 16 to 31 pairs (2 or 3 sequences of 8 KV heads) the workgroups that share a CU overlap their
// fixed costs, so only the tiles count twice there: (tiles per wavefront + 1) + (workgroups per CU - 1) x
// tiles per wavefront, fewer tiles per wavefront on a tie (3 sequences, K = 2048: 288 workgroups 12.7 -> 408
// workgroups 10.4; K = 4096: 17.5 -> 14.7; K = 8192: 29.7 -> 25.2; 2 sequences, K = 4096: 272 workgroups
// 13.9 -> 192 or 256 workgroups 12.3; K = 8192: 22.1 -> 18.1 - 18.4; K = 2048 stays at 272 workgroups, 9.8).
// The rows decoded since the refresh: a workgroup of their own (*tail_own = 1) or one wavefront's extra tile at the
// end (0), whichever the same estimate likes better; without their workgroups the launch can be exactly one
// workgroup per CU (16 sequences of 8 KV heads: K = 2048, 2 workgroups per pair and no tail workgroup, 256 in all,
// 28.7 us against 3 + 1, 512 in all, 32.6; K = 1024: 17.5 against 18.3; 8 sequences, K = 2048: 4 per pair 19.4
// against 20.0).  tail_rows > 128 (or no selected rows): all rows are shared out alike.
static inline int batched_tagged_workgroups(int64_t rows, int64_t tail_rows, int* tail_own, int64_t n_problems) {
    const bool small_tail = rows > 0 && tail_rows > 0 && tail_rows <= kMinChunk;
    const int64_t main_rows = small_tail ? rows : rows + tail_rows;
    const int64_t stretches = (main_rows + kMinChunk - 1) / kMinChunk;
    const int64_t tiles = (main_rows + 31) / 32;
    const bool few = n_problems < 32;
    int64_t best = 1, best_cost = -1, best_rounds = 0;
    int best_tail = 0;
    for (int tail = small_tail ? 1 : 0; tail >= 0; --tail) {
        for (int64_t n = 1; n <= stretches && n <= kMergeChunks; ++n) {
            const int64_t per_cu = ((n + tail) * n_problems + kComputeUnits - 1) / kComputeUnits;
            const int64_t rounds = (tiles + 4 * n - 1) / (4 * n);
            const int64_t fixed = 1 + (n + tail - 1) / 20;
            const int64_t extra = (small_tail && !tail) ? 1 : 0;          // the tail as one wavefront's last tile
            const int64_t cost = (few ? rounds + fixed + (per_cu - 1) * rounds : per_cu * (rounds + fixed)) + extra;
            if (best_cost < 0 || cost < best_cost || (few && cost == best_cost && tail == best_tail && rounds < best_rounds)) {   // ties (few pairs): fewer tiles per wavefront
                best = n; best_cost = cost; best_rounds = rounds; best_tail = tail;
            }
        }
    }
    *tail_own = best_tail;
    return (int)best;
}

// The same where the partial results are merged by slices (every workgroup its share: see attn_split_kernel) and
// the launch has at most 8 (sequence, KV head) pairs.  That merge costs a workgroup about the same whatever the
// number of partial results (a lane reads a quarter of them), so the tiles per wavefront decide: as many workgroups
// as give every wavefront the fewest tiles, within what the merge takes (`limit` partial results per pair) and what
// is resident at once (two workgroups per compute unit); the fewest workgroups among those.  A few rows decoded
// since the refresh (tail_rows <= 128) do not count: they get a workgroup of their own (*tail_own = 1) unless that
// one more partial result would cost every wavefront a tile; then one wavefront takes them as a second tile
// (K = 8192, one sequence of 8 KV heads: 64 workgroups 11.2 us, 63 + 1: 13.6, the ticketed form with 32: 12.3;
// 4 KV heads of 7 query heads: 10.1 / 10.7 / 12.8).  Measured against the sizing above, us per partial step, one
// sequence: 8 KV heads, K = 3072: 8.8 -> 7.4, 6144: 11.0 -> 10.0, 12288: 17.1 -> 14.9, 16384: 21.5 -> 18.8;
// 4 KV heads of 7: K = 3072: 8.8 -> 7.4, 4096: 9.0 -> 7.7, 6144: 11.2 -> 8.7, 8192: 12.7 -> 10.3.  (With 12 pairs
// it was no gain: 3 sequences of 4 KV heads, K = 8192: 15.3 -> 16.2.)
static inline int sliced_split_workgroups(int64_t rows, int64_t tail_rows, int* tail_own, int64_t n_problems, int limit) {
    const int64_t problems = n_problems > 0 ? n_problems : 1;
    int64_t cap = 2 * kComputeUnits / problems;
    if (cap > limit) cap = limit;
    if (cap < 1) cap = 1;
    const bool small_tail = rows > 0 && tail_rows <= kMinChunk;
    const int64_t tiles = ((small_tail ? rows : rows + tail_rows) + 31) / 32;
    auto rounds = [&](int64_t n) { return (tiles + 4 * n - 1) / (4 * n); };
    auto fewest = [&](int64_t upto) { int64_t n = upto; while (n > 1 && rounds(n - 1) == rounds(upto)) --n; return n; };
    *tail_own = (small_tail && cap > 1 && rounds(cap - 1) == rounds(cap)) ? 1 : 0;
    const int64_t n = fewest(*tail_own ? cap - 1 : cap);
    // (the tail's workgroups would be the only ones beyond one per compute unit: they wait for a unit to come free)
    if (*tail_own && n * problems <= kComputeUnits && (n + 1) * problems > kComputeUnits) *tail_own = 0;
    return (int)n;
}

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr int kBatchLayers = 32;         // layers one batched launch (rk_refresh_batched) takes; more go in several launches
constexpr int kHistBins = 2048;          // first-level histogram of the selection: top 11 key bits
constexpr int kMaxCandidates = 16384;    // most candidates the fast selection path sorts in LDS
constexpr int kHistShift = 32 - 11;      // key bits below the first-level histogram bin
constexpr int kPoolTile = 512;           // positions one workgroup pools and histograms ...
constexpr int kPoolTileLong = 1024;      // ... over rows of kPoolLongFrom positions or more: there the chip is full
constexpr int kPoolLongFrom = 98304;     // anyway and fewer, larger tiles win (per call at 131072 positions: selection
                                         // 38.2 -> 35.6 us, full step with selection 151.7 -> 144.9; at 32k and 64k
                                         // larger tiles lose: 17.4 -> 18.4 and 21.6 -> 22.2 us)
static inline int pool_tile_for(int64_t max_len) { return max_len >= kPoolLongFrom ? kPoolTileLong : kPoolTile; }

// Candidate slots per (sequence, KV head) of the selection: the K winners plus the rest of the
// histogram bin that holds the K-th score.
static inline int topk_cand_cap(int64_t k) {
    int64_t c = 1024;
    while (c < 2 * k && c < kMaxCandidates) c *= 2;
    return (int)c;
}

// Device workspace, carved in this order (every region 256-byte aligned).  The regions up to and
// including tag_rows must be zero when a workspace is first used (rk_workspace_init clears the
// whole workspace once); the counters and histograms are left cleared by the kernels that use
// them, the call numbers and tags only ever grow.  Where these regions lie depends on the
// geometry alone, never on max_len or max_k.
//   counters  int32 [B*Hkv][kCounterStride]  arrival tickets of the split attention kernel, one per
//                                            128-byte line
//   sel_counters int32 [B*Hkv][2]            listed candidates and arrival tickets of the selection
//   epochs    uint32 [B*Hkv]                 call number of the last merge inside a split kernel
//   hist      uint32 [B*Hkv][kHistBins]      first-level histogram of the pooled scores
//   tag_rows  16 B  [B*Hkv][kTagSlots][G*44]  tagged partial results of the kernels that merge
//                                            inside the launch (see merge_tagged in rk_attn.hip)
//   lse       fp32  [B*Hq]                   log-sum-exp when the caller does not ask for it
//   part_ml   fp32  [B*Hkv][kMaxChunks][G][2] running max and sum of every partial result
//   part_o    fp32  [B*Hkv][nch][G][128]     unnormalised partial outputs
//   pooled    fp32  [B*Hkv][max_len up to a multiple of 4]   group-max, pooled scores of the selection
//   scores    fp32  [B*Hq][max_len up to a multiple of 4]    raw scores between the two kernels of
//                                                            rk_full_attn_select
constexpr int kCounterStride = 32;       // int32 between two arrival counters: one 128-byte line each
constexpr int kTagDataRows = 43;          // a head's 128 output dims as rows of three (the last one holds two) ...
constexpr int kTagRowsPerHead = kTagDataRows + 1;   // ... plus the row with the chunk's log-sum-exp (see merge_tagged_heads)
constexpr int kTagSlots = kMergeChunks + 1;   // tagged partial results per (sequence, KV head): the chunks + the tail's own
struct Workspace {
    int32_t* counters;
    int32_t* sel_counters;
    uint32_t* epochs;
    uint32_t* hist;
    uint32_t* tag_rows;
    float* lse;
    float* part_ml;
    float* part_o;
    float* pooled;
    float* scores;
    uint64_t* cand_list;  // [B*Hkv][cand_cap] candidates (score image, ~position) of the spread-out selection;
                          // last, because its size depends on k
    int cand_cap;         // candidate slots the selection sorts in LDS
    int max_chunks;       // nch above
    size_t total;
};

// Row stride of the pooled-score area: rows are read with 16-byte loads.
static inline int64_t pooled_row_stride(int64_t max_len) { return (max_len + 3) / 4 * 4; }

// Bytes of the regions that must be zero at first use (the head of the workspace).
static inline size_t zero_kept_bytes(const rk_geom* g) {
    const size_t problems = (size_t)g->batch * g->n_kv_heads;
    const size_t G = (size_t)(g->n_q_heads / g->n_kv_heads);
    size_t off = problems * ((size_t)kCounterStride + 2 + 1 + (size_t)kHistBins) * sizeof(int32_t);
    off = (off + 255) / 256 * 256;
    return off + problems * kTagSlots * G * kTagRowsPerHead * 16;
}

static inline int max_chunks_for(int64_t max_len) {
    int64_t n = (max_len + kMinChunk - 1) / kMinChunk;
    if (n > kMaxChunks) n = kMaxChunks;
    if (n < 1) n = 1;
    return (int)n;
}

// Workgroups per (sequence, KV head) of the score-emitting split kernel of a full step (the
// finishing kernels must be told the same number).  The launch aims at about four tiles of 32 rows
// per wavefront, in whole multiples of the 256 CUs, between one and four workgroups per CU.
// Measured on the kernel alone, total workgroups -> us per launch (8 KV heads unless noted):
//   32778 rows:            256 -> 25.8, 512 -> 24.8 - 25.2, 768 -> 25.7 - 26.2, 1024 -> 25.6 - 25.7
//   65546 rows, 4 heads:   256 -> 28.5, 512 -> 27.6, 768 -> 28.6 - 28.9, 1024 -> 29.0 - 29.4
//   131082 rows:           256 -> 103.0, 512 -> 102.4 - 102.9, 768 -> 102.5, 1024 -> 100.1
// (384 workgroups, uneven over the CUs: 28.8 / 32.8 / 115.3.)  Few tiles per wavefront leave the
// launch's fixed costs (start, the merge across the wavefronts, the partial results) a larger share
// and make a ragged last round (2.67 tiles per wavefront with 768 workgroups at 32k rows) cost more;
// long rows want more loads in flight.
static inline int emit_split_workgroups(const rk_geom* g, int64_t max_len) {
    const int64_t problems = (int64_t)g->batch * g->n_kv_heads;
    const int64_t tiles = (max_len + 31) / 32 * problems;
    int64_t target = (tiles / 16 + kComputeUnits / 2) / kComputeUnits * kComputeUnits;      // 16 tiles per workgroup: 4 per wavefront
    if (target < kComputeUnits) target = kComputeUnits;
    if (target > 4 * kComputeUnits) target = 4 * kComputeUnits;
    return split_workgroups(max_len, problems, kMaxChunks, (int)target);
}

static inline Workspace carve(const rk_geom* g, int64_t max_len, int64_t max_k, void* base) {
    Workspace w;
    const size_t problems = (size_t)g->batch * g->n_kv_heads;
    const size_t G = (size_t)(g->n_q_heads / g->n_kv_heads);
    w.max_chunks = max_chunks_for(max_len);
    char* p = (char*)base;
    size_t off = 0;
    w.counters = (int32_t*)(p + off); off += problems * kCounterStride * sizeof(int32_t);
    w.sel_counters = (int32_t*)(p + off); off += 2 * problems * sizeof(int32_t);
    w.epochs = (uint32_t*)(p + off);  off += problems * sizeof(uint32_t);
    w.hist = (uint32_t*)(p + off);    off += problems * kHistBins * sizeof(uint32_t);
    off = align_up(off, 256);
    w.tag_rows = (uint32_t*)(p + off); off += problems * kTagSlots * G * kTagRowsPerHead * 16;
    w.lse = (float*)(p + off);        off += align_up((size_t)g->batch * g->n_q_heads * sizeof(float), 256);
    w.part_ml = (float*)(p + off);    off += align_up(problems * kMaxChunks * G * 2 * sizeof(float), 256);
    w.part_o = (float*)(p + off);     off += align_up(problems * w.max_chunks * G * kD * sizeof(float), 256);
    w.pooled = (float*)(p + off);     off += align_up(problems * (size_t)pooled_row_stride(max_len > 0 ? max_len : 1) * sizeof(float), 256);
    w.scores = (float*)(p + off);     off += align_up((size_t)g->batch * g->n_q_heads * (size_t)pooled_row_stride(max_len > 0 ? max_len : 1) * sizeof(float), 256);
    w.cand_cap = topk_cand_cap(max_k > 0 ? max_k : 1);
    w.cand_list = (uint64_t*)(p + off); off += align_up(problems * (size_t)w.cand_cap * sizeof(uint64_t), 256);
    w.total = off;
    return w;
}

static inline int check_geom(const rk_geom* g) {
    if (!g) return RK_ERR_INVALID_ARG;
    if (g->batch <= 0 || g->n_q_heads <= 0 || g->n_kv_heads <= 0) return RK_ERR_INVALID_ARG;
    if (g->n_q_heads % g->n_kv_heads != 0) return RK_ERR_INVALID_ARG;
    if (g->head_dim != kD) return RK_ERR_UNSUPPORTED;
    if (g->n_q_heads / g->n_kv_heads > RK_MAX_GROUP) return RK_ERR_UNSUPPORTED;
    if (g->batch > 65535 || g->n_kv_heads > 65535) return RK_ERR_UNSUPPORTED;
    return RK_OK;
}

static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

static inline int check_kv(const rk_kv& c, bool need_v = true) {
    if (!c.k || (need_v && !c.v)) return RK_ERR_INVALID_ARG;
    if (!aligned16(c.k) || !aligned16(c.v)) return RK_ERR_INVALID_ARG;
    // row indices are int32 and the kernels step past the end by up to kMaxChunks * kMinChunk rows
    if (c.stride_b < 0 || c.stride_h < 0 || c.capacity <= 0 || c.capacity > INT32_MAX - 2 * kMaxChunks * kMinChunk) return RK_ERR_INVALID_ARG;
    if (c.stride_b % 8 != 0 || c.stride_h % 8 != 0) return RK_ERR_INVALID_ARG;
    if (c.stride_b >= (1ll << 56)) return RK_ERR_UNSUPPORTED;   // the top byte of the sequence stride travels as a flag to the kernels
    if (c.stride_h > INT32_MAX) return RK_ERR_UNSUPPORTED;      // the head stride travels as 32 bits to the kernels
    return RK_OK;
}

static inline int check_workspace(const rk_geom* g, int64_t max_len, int64_t max_k, void* ws,
                                  size_t bytes, Workspace* out) {
    if (!ws || ((uintptr_t)ws & 255u) != 0) return RK_ERR_WORKSPACE;
    *out = carve(g, max_len, max_k, ws);
    if (bytes < out->total) return RK_ERR_WORKSPACE;
    return RK_OK;
}

static inline int launch_status() {
    return hipGetLastError() == hipSuccess ? RK_OK : RK_ERR_HIP;
}

// Stages shared by the entry points (arguments already checked by the caller).
//   full_attn_stage: the split kernel, then either the merge inside it (no weights), the merge +
//     normalise kernel (weights in place), or, with pool_half >= 0, the fused finish that also
//     leaves the pooled group scores and their histogram in the workspace.  no_v: the split kernel
//     is the scores-only one (K rows only; out must be NULL, pool_half >= 0).  co_run: the launch is
//     shaped for running beside another stream's kernels (see split_workgroups).  defer_pool (with
//     pool_half >= 0 and out != NULL): only the output is finished; the raw scores and the chunk
//     statistics stay in the workspace for pool_batched_stage, which does for several layers at
//     once what the finishing kernel's pooling tiles do for one.
//   select_stage: top-K over the pooled scores and histogram that are in the workspace.
__attribute__((visibility("hidden")))
int full_attn_stage(const rk_geom* geom, const void* q, rk_kv full, const int32_t* seq_lens, int32_t max_len,
                    void* out, float* weights, int64_t w_stride, float* lse, const int32_t* pred, int32_t pred_val,
                    const Workspace& ws, hipStream_t st, bool scores_only, int pool_half, bool no_v, int agg,
                    bool co_run = false, bool defer_pool = false);
__attribute__((visibility("hidden")))
int pool_batched_stage(const rk_geom* geom, int n_layers, const Workspace* wss, const int32_t* seq_lens, int32_t max_len,
                       int64_t full_capacity, int pool_half, int agg, const int32_t* const* pred, int32_t pred_val,
                       hipStream_t st);
//   gather_stage: rk_gather_small_kv plus an optional per-sequence count of refreshes.
__attribute__((visibility("hidden")))
int gather_stage(const rk_geom* geom, rk_kv full, const int32_t* idx, int32_t k, rk_kv small,
                 const int32_t* seq_lens, int32_t* tail_start, int32_t* n_refresh,
                 const int32_t* pred, int32_t pred_val, hipStream_t stream);
//   pool_stage: group aggregation, max-pool and histogram of normalised per-head scores (first
//     kernel of rk_topk_select); check_select_args: the limits on k, pool_w and agg.
__attribute__((visibility("hidden")))
int pool_stage(const rk_geom* geom, const float* weights, int64_t w_stride, const int32_t* seq_lens,
               int32_t max_len, int32_t pool_w, int32_t agg, const int32_t* pred, int32_t pred_val,
               const Workspace& ws, hipStream_t st);
__attribute__((visibility("hidden")))
int check_select_args(int32_t k, int32_t pool_w, int32_t agg, int32_t max_len);
__attribute__((visibility("hidden")))
int select_stage(const rk_geom* geom, const int32_t* seq_lens, int32_t max_len, int32_t k, int32_t* idx,
                 float* sel_scores, const int32_t* pred, int32_t pred_val, const Workspace& ws, hipStream_t st);

// Batched forms for rk_refresh_batched: the selections, then the gathers, of up to kBatchLayers
// layers in one launch each.  wss[l] holds what rk_full_attn_pool left for layer l.
__attribute__((visibility("hidden")))
int select_batched_stage(const rk_geom* geom, int n_layers, const Workspace* wss, int32_t* const* idx,
                         const int32_t* seq_lens, int32_t max_len, int32_t k, const int32_t* const* pred, int32_t pred_val,
                         hipStream_t st);
__attribute__((visibility("hidden")))
int gather_batched_stage(const rk_geom* geom, int n_layers, const rk_kv* full, const rk_kv* small, int32_t* const* idx,
                         int32_t k, const int32_t* seq_lens, int32_t* const* tail_start, int32_t* const* n_refresh,
                         const int32_t* const* pred, int32_t pred_val, hipStream_t st);

}  // namespace rk
