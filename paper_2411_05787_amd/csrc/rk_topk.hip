// rk_topk_select for gfx950: group max + max-pool, then an exact, tie-correct top-K.
//
// The order is decided on the order-preserving 32-bit image of the pooled score P (integer
// compares only, so the result is exact): larger image first, equal images by lower position.
//
// Kernel 1, whole chip (pool_hist_kernel; tiles of 512 positions, of 1024 from 98304 positions on):
//   P[j] = max over the G heads of the group and over the pooling window, staged through LDS so
//   that every weight is read once; P is stored and its top 11 image bits are histogrammed (LDS,
//   then one global atomic per non-empty bin).
// Kernel 2 (select_kernel), workgroups of 1024 threads: from the histogram, the bin b1 that holds
//   the K-th largest score; every position in that bin or a higher one is a candidate (the K
//   winners plus the rest of one bin).  What is listed and ranked are runs of candidates: up to
//   four neighbours with the same pooled score (the pooling window makes neighbours equal, so runs
//   are several times fewer than positions).  The runs are packed into a dense list: for rows up
//   to 8192 positions by the one workgroup of the (sequence, KV head), in LDS; for longer rows by
//   one workgroup per 4096 positions (per 32768 in a launch over many long rows), into the
//   workspace (one atomic add per workgroup reserves the space), and the workgroup that arrives
//   last goes on alone.  It takes the list into registers and bucket-sorts it back into LDS on the
//   64-bit item (P image, position, length): 2048 buckets from the lowest candidate image up to
//   the bin of the 64-th largest score (of equal width, or laid out from the histogram), one more
//   bucket for everything above (fewer than 64 positions); a scan turns bucket counts into
//   offsets, and the rank of a run's first position is the number of positions in the buckets
//   above plus those of the larger runs in its own bucket (a few compares).  Positions that rank
//   below K' are written out directly: idx comes out in rank order.  The kernel also clears the
//   histogram for the next call.
// Dense or degenerate score distributions take further exact steps in kernel 2 (one workgroup):
// more runs than fit in LDS -> bin b1 is cut once more by the next 11 image bits (one more pass
// over P) and only its upper part stays a candidate; a bucket with more than 1024 runs -> the list
// is bitonic-sorted instead of ranked; still too many candidates (e.g. all scores equal) -> a last
// radix pass (10 bits) finds the K-th largest image T exactly, positions with P > T and the first
// positions with P == T are collected in position order, then bitonic-sorted.
#include "rk_internal.h"
#include "rk_device.h"

namespace rk {

constexpr int kSelThreads = 1024;
constexpr int kSelTile = 4 * kSelThreads;                // positions per workgroup when the selection is spread out
constexpr int kSelSingle = 2 * kSelTile;                 // rows up to this length are left to one workgroup
constexpr int kSelHeld = 8 * kSelTile;                   // positions a workgroup keeps in registers (NV vectors per thread)
constexpr int kBatchSingleFrom = 64;                     // ... and so are all rows of a batched launch with this many rows
constexpr int kBuckets = 2048;                           // regular buckets, plus one for all above
constexpr int kBucketLimit = 1024;                       // larger buckets: sort instead of ranking
constexpr int kAdaptiveFrom = 8192;                      // candidates from which buckets follow the histogram
constexpr int kTopLoose = 64;                            // scores above the bucketed range: fewer than this
constexpr int kListTry = 4;                              // runs are listed for up to this many times cand_cap positions
static_assert(kHistBins == 1 << 11, "first-level histogram is 11 bits wide");
static_assert(kHistBins == 2 * kSelThreads, "the selection scans the histogram two bins per thread");

// What is ranked is a run: up to kRunMax positions next to each other with the same pooled score
// (the pooling window makes the scores of up to pool_w neighbours equal, so there are several
// times fewer runs than candidate positions, and the ranking costs the square of a bucket's
// size).  A run is one 64-bit item: score image | kPosTop - first position | length - 1; larger
// items come first in the selection (two runs never share a first position, so the length never
// decides), and the positions of a run follow each other in the output.
constexpr int kRunMax = 4;                               // a run lies inside one 16-byte vector of scores
constexpr uint32_t kPosTop = (1u << 28) - 1u;            // positions are below RK_MAX_SELECT_LEN = 2^28
static_assert(RK_MAX_SELECT_LEN == (int64_t)kPosTop + 1, "28 bits of an item hold the position");
__device__ __forceinline__ uint64_t item_of(uint32_t key, int j, int len = 1) {
    return ((uint64_t)key << 32) | (uint64_t)(((kPosTop - (uint32_t)j) << 4) | (uint32_t)(len - 1));
}
__device__ __forceinline__ int item_pos(uint64_t item) { return (int)(kPosTop - ((uint32_t)item >> 4)); }
__device__ __forceinline__ uint32_t item_len(uint64_t item) { return ((uint32_t)item & 15u) + 1u; }

template <int TILE>
__global__ __launch_bounds__(256)
void pool_hist_kernel(const float* __restrict__ weights, int64_t w_stride, const int32_t* seq_lens,
                      int32_t max_len, int32_t Hq, int32_t Hkv, int32_t G, int32_t half, int32_t agg,
                      float* __restrict__ pooled, int64_t pooled_stride, uint32_t* __restrict__ hist,
                      const int32_t* pred, int32_t pred_val) {
    const int g = blockIdx.y, b = blockIdx.z;
    if (pred != nullptr && pred[b] != pred_val) return;
    const int len = min(seq_lens[b], max_len);
    const int j0 = blockIdx.x * TILE;
    if (j0 >= len) return;
    __shared__ float sA[TILE + RK_MAX_POOL_W - 1];
    __shared__ uint32_t sH[kHistBins];
    const float* wg = weights + ((int64_t)b * Hq + (int64_t)g * G) * w_stride;
    const int span = TILE + 2 * half;
    for (int i = threadIdx.x; i < kHistBins; i += 256) sH[i] = 0;
    for (int i = threadIdx.x; i < span; i += 256) {
        const int j = j0 - half + i;
        float a = -INFINITY;                     // outside [0, len): never wins a max
        if (j >= 0 && j < len) {
            for (int gi = 0; gi < G; ++gi) a = aggregate(a, wg[(int64_t)gi * w_stride + j], gi, agg);
            if (agg == RK_AGG_MEAN) a = __fdiv_rn(a, (float)G);
        }
        sA[i] = a;
    }
    __syncthreads();
    const int64_t bg = (int64_t)b * Hkv + g;
    float* out = pooled + bg * pooled_stride;
    for (int i = threadIdx.x; i < TILE; i += 256) {
        const int j = j0 + i;
        if (j < len) {
            float m = sA[i];
            for (int d = 1; d <= 2 * half; ++d) m = fmaxf(m, sA[i + d]);
            m += 0.0f;                           // -0 becomes +0: one bit pattern per value
            out[j] = m;
            atomicAdd(&sH[key_of(m) >> kHistShift], 1u);
        }
    }
    __syncthreads();
    uint32_t* gh = hist + bg * kHistBins;
    for (int i = threadIdx.x; i < kHistBins; i += 256) {
        const uint32_t c = sH[i];
        if (c != 0) atomicAdd(&gh[i], c);
    }
}

// Inclusive prefix sum over the NT threads of the workgroup, in thread order.  `scratch` holds
// NT / 64 words.  Returns the inclusive sum; *total gets the workgroup sum.
template <int NT>
__device__ __forceinline__ uint32_t block_inclusive_scan(uint32_t v, uint32_t* scratch, uint32_t* total) {
    constexpr int NWV = NT / 64;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    // inside the wavefront: a scan of every row of 16 lanes on the DPP path (a lane whose source
    // would lie outside its row adds 0), then the totals of the rows before, through scalar registers
    uint32_t x = v;
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xF, 0xF, true);     // row_shr:1
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xF, 0xF, true);     // row_shr:2
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xF, 0xF, true);     // row_shr:4
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xF, 0xF, true);     // row_shr:8
    {
        const uint32_t t0 = (uint32_t)__builtin_amdgcn_readlane((int)x, 15), t1 = (uint32_t)__builtin_amdgcn_readlane((int)x, 31);
        const uint32_t t2 = (uint32_t)__builtin_amdgcn_readlane((int)x, 47);
        const int row = lane >> 4;
        x += row == 0 ? 0u : row == 1 ? t0 : row == 2 ? t0 + t1 : t0 + t1 + t2;
    }
    __syncthreads();                              // scratch may still be read from a previous scan
    if (lane == 63) scratch[w] = x;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NWV; ++i) {
        const uint32_t s = scratch[i];
        if (i < w) base += s;
        tot += s;
    }
    *total = tot;
    return x + base;
}

// Inclusive prefix sum over the 64 lanes of the wavefront (the first half of the scan above).
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
    const int lane = threadIdx.x & 63;
    uint32_t x = v;
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xF, 0xF, true);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xF, 0xF, true);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xF, 0xF, true);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xF, 0xF, true);
    const uint32_t t0 = (uint32_t)__builtin_amdgcn_readlane((int)x, 15), t1 = (uint32_t)__builtin_amdgcn_readlane((int)x, 31);
    const uint32_t t2 = (uint32_t)__builtin_amdgcn_readlane((int)x, 47);
    const int row = lane >> 4;
    return x + (row == 0 ? 0u : row == 1 ? t0 : row == 2 ? t0 + t1 : t0 + t1 + t2);
}

// Given a histogram of NB bins (LDS or global) find the bin that holds the kk-th largest entry,
// counting from the top bin down: sOut[0] = that bin, sOut[1] = entries in higher bins.
// All NT threads call; the result is valid after the call (it ends with a barrier).
template <int NT, int NB>
__device__ void find_bin_from_top(const uint32_t* hist, uint32_t kk, uint32_t* sScan, uint32_t* sOut) {
    constexpr int BPT = NB / NT;
    static_assert(BPT >= 1 && BPT * NT == NB, "bins divide evenly over the threads");
    const int rt = NT - 1 - (int)threadIdx.x;       // thread 0 owns the top bins
    uint32_t h[BPT];
    uint32_t local = 0;
#pragma unroll
    for (int i = 0; i < BPT; ++i) { h[i] = hist[rt * BPT + i]; local += h[i]; }
    uint32_t total;
    const uint32_t incl = block_inclusive_scan<NT>(local, sScan, &total);   // entries in bins >= BPT*rt
    uint32_t above = incl - local;
    if (above < kk && kk <= incl) {
#pragma unroll
        for (int i = BPT - 1; i >= 0; --i) {
            if (above + h[i] >= kk) { sOut[0] = (uint32_t)(rt * BPT + i); sOut[1] = above; break; }
            above += h[i];
        }
    }
    __syncthreads();
}

// One histogram pass of the slow-path radix select.  On entry the keys still in play are those
// with (key & mask) == prefix and the kk-th largest of them is wanted.  Bins are BITS wide at
// `shift`.  Result in sOut as for find_bin_from_top.
template <int BITS>
__device__ void radix_pass(const float* __restrict__ P, int n, uint32_t prefix, uint32_t mask, int shift,
                           uint32_t kk, uint32_t* sHist, uint32_t* sScan, uint32_t* sOut) {
    constexpr int NB = 1 << BITS;
    const int tid = threadIdx.x;
    for (int i = tid; i < NB; i += kSelThreads) sHist[i] = 0;
    __syncthreads();
    // 16-byte loads, eight of them in flight per thread (rows start 16-byte aligned and are padded
    // to a multiple of four scores); few keys match the prefix, so the atomics are sparse
    const float4* P4 = reinterpret_cast<const float4*>(P);
    const int nvec = (n + 3) >> 2;
    auto count = [&](float v, int j) {
        const uint32_t key = key_of(v);
        if (j < n && (key & mask) == prefix) atomicAdd(&sHist[(key >> shift) & (NB - 1)], 1u);
    };
    constexpr int UN = 8;
    for (int v0 = 0; v0 < nvec; v0 += kSelThreads * UN) {
        float4 pv[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int v = v0 + u * kSelThreads + tid;
            pv[u] = v < nvec ? P4[v] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int v = v0 + u * kSelThreads + tid;
            const int j = v < nvec ? v << 2 : n;
            count(pv[u].x, j); count(pv[u].y, j + 1); count(pv[u].z, j + 2); count(pv[u].w, j + 3);
        }
    }
    __syncthreads();
    find_bin_from_top<kSelThreads, NB>(sHist, kk, sScan, sOut);
}

// Sorts sKeys[0 .. npad) descending (npad a power of two); all kSelThreads threads call.
// Wavefront w owns the compare-exchange pairs [w * PW, (w + 1) * PW), PW = npad / 2 / 16.  For a
// stride <= PW those pairs only touch the wavefront's own 2 * PW elements, so such stages are
// separated by a wavefront-local ordering of LDS traffic; only the strides above PW (10 of the
// 78 stages at npad = 4096) need a workgroup barrier.
__device__ void bitonic_sort_desc(uint64_t* sKeys, int npad) {
    constexpr int NWV = kSelThreads / 64;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int half = npad >> 1;
    if (half < kSelThreads) {
        // small lists: one pair per thread at most, plain barriers
        for (int size = 2; size <= npad; size <<= 1) {
            for (int stride = size >> 1; stride > 0; stride >>= 1) {
                if (tid < half) {
                    const int lo = ((tid & ~(stride - 1)) << 1) | (tid & (stride - 1));
                    const int hi = lo + stride;
                    const bool desc = (lo & size) == 0;
                    const uint64_t a = sKeys[lo], c = sKeys[hi];
                    if ((a < c) == desc) { sKeys[lo] = c; sKeys[hi] = a; }
                }
                __syncthreads();
            }
        }
        return;
    }
    const int PW = half / NWV;                    // pairs per wavefront, a multiple of 64
    bool need_barrier = false;                    // the previous stage crossed wavefront blocks
    for (int size = 2; size <= npad; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            const bool cross = stride > PW;
            if (cross || need_barrier) __syncthreads(); else wave_lds_sync();
            for (int i = w * PW + lane; i < (w + 1) * PW; i += 64) {
                const int lo = ((i & ~(stride - 1)) << 1) | (i & (stride - 1));
                const int hi = lo + stride;
                const bool desc = (lo & size) == 0;
                const uint64_t a = sKeys[lo], c = sKeys[hi];
                if ((a < c) == desc) { sKeys[lo] = c; sKeys[hi] = a; }
            }
            need_barrier = cross;
        }
    }
    __syncthreads();
}

// Grid (tiles, KV heads, sequences).  With one tile the workgroup does everything.  With more,
// every workgroup derives the thresholds from the histogram, packs the runs of candidates among
// its own tile_vecs * kSelTile positions into a list in the workspace (one atomic add per
// workgroup reserves the space), and the workgroup that arrives last (ticket, as in the attention
// kernels) takes the list into registers and ranks it: the pass over all positions, which is what
// a single workgroup spends most of its time on, is spread over the chip.
// The selection of one (sequence b, KV head blockIdx.y), by the workgroups blockIdx.x = 0 .. gridDim.x - 1.
template <bool ADAPT>                    // ADAPT: compiled with the histogram-driven bucket layout (large K only)
__device__ __forceinline__
void select_body(const float* __restrict__ pooled, int64_t pooled_stride, const int32_t* seq_lens,
                 int32_t max_len, int32_t k, uint32_t* __restrict__ hist, int32_t cand_cap,
                 int32_t* __restrict__ idx, float* __restrict__ sel_scores,
                 const int32_t* pred, int32_t pred_val,
                 int32_t* __restrict__ sel_counters, uint64_t* __restrict__ cand_list, const int b,
                 const int tile_vecs) {
    const int tile = blockIdx.x, g = blockIdx.y, Hkv = gridDim.y;
    const bool multi = gridDim.x > 1;
    if (pred != nullptr && pred[b] != pred_val) return;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint64_t* sKeys = reinterpret_cast<uint64_t*>(smem);                   // [cand_cap]
    uint32_t* sHist = reinterpret_cast<uint32_t*>(sKeys + cand_cap);       // [2 * (kBuckets + 1)]: bucket
                                                                           // arrays, or the radix histogram
    uint32_t* sScan = sHist + 2 * (kBuckets + 1);                          // [16]
    uint32_t* sOut = sScan + kSelThreads / 64;                             // [4]
    uint32_t* sCount = sOut + 4;                                           // [1]
    uint16_t* sTab = reinterpret_cast<uint16_t*>(sCount + 1);              // [kHistBins] buckets of each first-level bin
                                                                           // (allocated only if cand_cap > kAdaptiveFrom)

    const int tid = threadIdx.x;
    const int n = min(seq_lens[b], max_len);
    const int kprime = min(k, max(n, 0));
    const int64_t bg = (int64_t)b * Hkv + g;
    const int64_t ob = bg * k;
    if (kprime <= 0) {                      // nothing was histogrammed for an empty sequence
        if (tile == 0)
            for (int i = tid; i < k; i += kSelThreads) { idx[ob + i] = -1; if (sel_scores) sel_scores[ob + i] = 0.f; }
        return;
    }
    const float* P = pooled + bg * pooled_stride;
    uint32_t* gh = hist + bg * kHistBins;

    // The first 32 scores of every thread (the whole row up to 32768 positions) are requested now,
    // 16-byte loads all in flight together with the histogram's, and stay in registers.
    constexpr int NV = kSelHeld / kSelTile;
    const float4* P4 = reinterpret_cast<const float4*>(P);
    const int nvec = (n + 3) >> 2;
    // positions at and beyond n read as -1: below every candidate threshold (scores are >= 0)
    auto load4 = [&](int v) -> float4 {
        float4 x = (v < nvec) ? P4[v] : make_float4(-1.f, -1.f, -1.f, -1.f);
        if (4 * v + 3 >= n && v < nvec) {             // the row's last, partial vector
            if (4 * v + 1 >= n) x.y = -1.f;
            if (4 * v + 2 >= n) x.z = -1.f;
            x.w = -1.f;
        }
        return x;
    };
    float4 held[NV];
    if (!multi) {
#pragma unroll
        for (int u = 0; u < NV; ++u) held[u] = load4(u * kSelThreads + tid);
    } else {
        // this workgroup's tile_vecs * kSelTile positions (tile_vecs is 1 or NV)
        held[0] = load4(tile * tile_vecs * kSelThreads + tid);
        if (tile_vecs > 1) {
#pragma unroll
            for (int u = 1; u < NV; ++u) held[u] = load4((tile * tile_vecs + u) * kSelThreads + tid);
        }
    }

    // From the histogram, in one scan from the top bin down (thread 0 owns the top two bins):
    // the bin b1 that holds the K'-th largest score (with the count above it), and the bin that
    // holds the kTopLoose-th largest, which bounds the bucketed range from above so that the one
    // bucket for "everything above" stays small (its items are ranked by a loop over the bucket).
    if (tid == 0) *sCount = 0;
    for (int i = tid; i < kBuckets + 1; i += kSelThreads) sHist[i] = 0;     // bucket sizes of the fast path
    uint32_t h0, h1;                         // this thread's two bins of the first-level histogram
    {
        const int rt = kSelThreads - 1 - tid;
        h0 = gh[2 * rt]; h1 = gh[2 * rt + 1];
        uint32_t total;
        const uint32_t incl = block_inclusive_scan<kSelThreads>(h0 + h1, sScan, &total);   // entries in bins >= 2 rt
        const uint32_t abv = incl - (h0 + h1);
        const uint32_t kk1 = (uint32_t)kprime, kk2 = min((uint32_t)kprime, (uint32_t)kTopLoose);
        if (abv < kk1 && kk1 <= incl) {
            const bool upper = abv + h1 >= kk1;
            sOut[0] = (uint32_t)(2 * rt + (upper ? 1 : 0));
            sOut[1] = upper ? abv : abv + h1;
            sOut[2] = upper ? h1 : h0;
        }
        if (abv < kk2 && kk2 <= incl) sOut[3] = (uint32_t)(2 * rt + (abv + h1 >= kk2 ? 1 : 0));
        if (!multi) { gh[2 * rt] = 0; gh[2 * rt + 1] = 0; }     // cleared for the next call
        __syncthreads();
    }
    const uint32_t b1 = sOut[0];
    const uint32_t above = sOut[1];
    uint32_t count_ge = above + sOut[2];
    const uint32_t key_top = (sOut[3] + 1u) << kHistShift;      // sOut[3] >= b1; wraps to 0 for the last bin

    uint32_t key_thr = b1 << kHistShift;
    // The list holds runs, so it may have room where the positions are too many: up to
    // kListTry * cand_cap positions the runs are listed anyway, counted as they are, and the list
    // is used if they fit.  (Bucket offsets below are counted in 16 bits: 65535 positions at most.)
    const bool try_list = count_ge <= (uint32_t)min(kListTry * cand_cap, 0xFFFF);    // the same in every workgroup of (b, g)
    bool listed = false;                    // the runs of all candidates are in the workspace

    // The runs of candidates inside one vector of four scores (positions j .. j + 3; a candidate is
    // a score >= thr; scores are >= +0 and -0 never occurs, so equal scores have equal bits and the
    // order-preserving image is the bit pattern with the top bit set): count_runs() counts them,
    // visit_runs() calls visit(image, first position, length) for each, in position order.
    auto count_runs = [](const float4 x, float thr) -> uint32_t {
        const uint32_t a = __float_as_uint(x.x), b = __float_as_uint(x.y), c = __float_as_uint(x.z), d = __float_as_uint(x.w);
        return (x.x >= thr ? 1u : 0u) + (x.y >= thr && b != a ? 1u : 0u) + (x.z >= thr && c != b ? 1u : 0u) +
               (x.w >= thr && d != c ? 1u : 0u);
    };
    auto visit_runs = [](const float4 x, int j, float thr, auto&& visit) {
        const uint32_t a = __float_as_uint(x.x), b = __float_as_uint(x.y), c = __float_as_uint(x.z), d = __float_as_uint(x.w);
        const int ed = d == c ? 1 : 0;                       // positions after j + 2 with its score
        const int ec = c == b ? 1 + ed : 0;                  // ... after j + 1
        const int eb = b == a ? 1 + ec : 0;                  // ... after j
        if (x.x >= thr) visit(a | 0x80000000u, j, 1 + eb);
        if (x.y >= thr && b != a) visit(b | 0x80000000u, j + 1, 1 + ec);
        if (x.z >= thr && c != b) visit(c | 0x80000000u, j + 2, 1 + ed);
        if (x.w >= thr && d != c) visit(d | 0x80000000u, j + 3, 1);
    };
    static_assert(kRunMax == 4, "runs are found inside one float4");

    uint32_t n_items = 0;                   // runs in the list
    if (multi) {
        int32_t* n_listed = sel_counters + bg * 2;
        int32_t* arrived = n_listed + 1;
        uint64_t* list = cand_list + bg * cand_cap;
        if (try_list) {
            const float t1 = value_of(key_thr);
            uint32_t c = count_runs(held[0], t1);
            if (tile_vecs > 1) {
#pragma unroll
                for (int u = 1; u < NV; ++u) c += count_runs(held[u], t1);
            }
            uint32_t total;
            const uint32_t incl = block_inclusive_scan<kSelThreads>(c, sScan, &total);
            if (tid == 0 && total != 0)
                *sCount = (uint32_t)__hip_atomic_fetch_add(n_listed, (int32_t)total, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            uint32_t pos = *sCount + incl - c;
            auto put = [&](uint32_t key, int j, int len) {
                if (pos < (uint32_t)cand_cap)                      // runs beyond the list's end are only counted
                    __hip_atomic_store(&list[pos], item_of(key, j, len), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ++pos;
            };
            visit_runs(held[0], (tile * tile_vecs * kSelThreads + tid) << 2, t1, put);
            if (tile_vecs > 1) {
#pragma unroll
                for (int u = 1; u < NV; ++u) visit_runs(held[u], ((tile * tile_vecs + u) * kSelThreads + tid) << 2, t1, put);
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // the list entries are acknowledged
        }
        __syncthreads();                                           // ... and every thread has read the histogram
        if (tid == 0) sOut[1] = (uint32_t)__hip_atomic_fetch_add(arrived, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (sOut[1] != gridDim.x - 1) return;
        // last to arrive: everything of this (b, g) is in (a workgroup has the answer of its
        // reservation before it writes its entries, hence before its ticket: the count is final);
        // leave the workspace clean, then rank
        if (tid == 0) {
            sOut[2] = (uint32_t)__hip_atomic_load(n_listed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(n_listed, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(arrived, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *sCount = 0;
        }
        { const int rt = kSelThreads - 1 - tid; gh[2 * rt] = 0; gh[2 * rt + 1] = 0; }
        __syncthreads();
        n_items = sOut[2];
        listed = try_list && n_items <= (uint32_t)cand_cap;
        if (!listed) {                                             // too many candidates: go on alone, from the scores
#pragma unroll
            for (int u = 0; u < NV; ++u) held[u] = load4(u * kSelThreads + tid);
        }
    }
    float thr = value_of(key_thr);                       // lowest candidate score (scores are >= 0)
    // The runs of candidates among NV vectors per thread (vector u of the thread is number
    // v0 + u * kSelThreads + tid of the row) go to the end of the list in sKeys: every wavefront
    // counts its own, reserves the room with one LDS atomic and writes them there.  The order of
    // the list depends on the order of the reservations; nothing after it depends on that order.
    auto list_candidates = [&](const float4 (&x)[NV], int v0) {
        uint32_t c = 0;
#pragma unroll
        for (int u = 0; u < NV; ++u) c += count_runs(x[u], thr);
        const uint32_t incl = wave_inclusive_scan(c);
        const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
        if (tot == 0) return;                                      // the same in all 64 lanes
        uint32_t base = 0;
        if ((tid & 63) == 63) base = atomicAdd(sCount, tot);
        uint32_t pos = (uint32_t)__builtin_amdgcn_readlane((int)base, 63) + incl - c;
#pragma unroll
        for (int u = 0; u < NV; ++u)
            visit_runs(x[u], (v0 + u * kSelThreads + tid) << 2, thr, [&](uint32_t key, int j, int len) {
                if (pos < (uint32_t)cand_cap) sKeys[pos] = item_of(key, j, len);    // runs beyond the end are only counted
                ++pos;
            });
    };
    // One pass over the row, which is the only work here that is proportional to n: the vectors
    // held in registers first, the rest of a longer row NV vectors per thread at a time, all of
    // them in flight together.  Returns the number of runs (they are in sKeys if they fit).
    bool held_is_row_start = true;
    auto list_row = [&]() -> uint32_t {
        if (!held_is_row_start) {
#pragma unroll
            for (int u = 0; u < NV; ++u) held[u] = load4(u * kSelThreads + tid);
        }
        list_candidates(held, 0);
        for (int v0 = NV * kSelThreads; v0 < nvec; v0 += kSelThreads * NV) {
#pragma unroll
            for (int u = 0; u < NV; ++u) held[u] = load4(v0 + u * kSelThreads + tid);
            list_candidates(held, v0);
            held_is_row_start = false;
        }
        __syncthreads();
        const uint32_t runs = *sCount;
        __syncthreads();
        if (tid == 0) *sCount = 0;
        return runs;
    };
    // Candidates are the positions whose image is >= key_thr.  Normally that is "bin b1 or above",
    // taken from the workspace (listed) or from the row; if their runs are too many for LDS, bin
    // b1 is cut once more by the next 11 image bits.
    uint32_t prefix = key_thr, mask = 0x7FFu << kHistShift, kk = (uint32_t)kprime - above;   // radix-select state
    bool refined = false;
    bool in_lds = false;                    // the runs of all candidates are in sKeys
    if (!listed && try_list && !multi) {    // (spread out and not listed: the runs were counted and do not fit)
        n_items = list_row();
        in_lds = n_items <= (uint32_t)cand_cap;
    }
    if (!listed && !in_lds) {               // (more than cand_cap positions: fewer would have been listed)
        radix_pass<11>(P, n, prefix, mask, 10, kk, sHist, sScan, sOut);
        const uint32_t b2 = sOut[0];
        count_ge = above + sOut[1] + sHist[b2];
        prefix |= b2 << 10; mask |= 0x7FFu << 10; kk -= sOut[1];
        key_thr = prefix;
        thr = value_of(key_thr);
        refined = true;
        __syncthreads();
        if (count_ge <= (uint32_t)cand_cap) {
            n_items = list_row();
            in_lds = true;
        }
    }
    // bucket width: the smallest power of two for which [key_thr, key_top) fits in kBuckets buckets
    const uint32_t span = key_top - 1u - key_thr;        // 11 significant bits are left after the shift
    const int bucket_shift = span >= (uint32_t)kBuckets ? 32 - 11 - __builtin_clz(span) : 0;

    // Buckets of the fast path.  Preferred layout: every first-level bin from b1 up to the bin of
    // the kTopLoose-th largest score gets a power-of-two number of equal-width buckets in
    // proportion to its count in the histogram, so that all buckets hold about the same number of
    // candidates however the scores are distributed over the octaves (scores thin out towards the
    // top: equal-width buckets over the whole range leave most candidates in the lowest few, and
    // the ranking below costs the square of a bucket's size).  sTab[bin] = first bucket | log2 of
    // the number of buckets << 11.  Used from kAdaptiveFrom candidates on (below that, building the
    // table costs more than it saves: measured).  Otherwise, and when the threshold is not on a bin
    // boundary or the bins need more than kBuckets buckets: equal-width buckets over the whole range.
    bool adaptive = false;
    auto bucket_of = [&](uint32_t key) -> uint32_t {
        if (ADAPT && adaptive) {
            if (key_top != 0u && key >= key_top) return (uint32_t)kBuckets;
            const uint32_t t = sTab[key >> kHistShift], e = t >> 11;
            return (t & 0x7FFu) + ((key >> (kHistShift - e)) & ((1u << e) - 1u));
        }
        return min((key - key_thr) >> bucket_shift, (uint32_t)kBuckets);
    };
    // The positions of a run whose first one has rank r, as far as they rank below K'.
    auto write_run = [&](uint64_t item, uint32_t r) {
        const int j = item_pos(item);
        const uint32_t len = min(item_len(item), (uint32_t)kprime - min(r, (uint32_t)kprime));
        for (uint32_t i = 0; i < len; ++i) {
            idx[ob + r + i] = j + (int)i;
            if (sel_scores) sel_scores[ob + r + i] = value_of((uint32_t)(item >> 32));
        }
    };
    int nvalid;                             // entries of sKeys that are real (sorting paths)
    if (listed || in_lds) {
        // ---- candidates = every position whose image is >= key_thr, count_ge of them ----
        // Their runs are in a dense list (in the workspace, put there by all the workgroups of the
        // row, or in LDS); everything from here on runs on the list: up to kItems items per thread,
        // taken into registers so that the same LDS array can receive them again sorted by bucket.
        // A bucket is counted twice in one word, runs << 16 | positions (neither field overflows:
        // at most cand_cap runs and 65535 positions in all).
        uint32_t* sCnt = sHist;                         // [kBuckets + 1] bucket sizes, then fill marks (in runs)
        uint32_t* sStart = sHist + kBuckets + 1;        // [kBuckets + 1] bucket offsets: runs << 16 | positions
        static_assert(kMaxCandidates < (1 << 16), "runs and positions of a bucket are counted in 16 bits each");
        if (refined) {                                  // the radix pass used the array: clear it again
            for (int i = tid; i < kBuckets + 1; i += kSelThreads) sCnt[i] = 0;
        }
        uint32_t total;
        if (ADAPT && !refined && count_ge > (uint32_t)kAdaptiveFrom) {
            const int rt = kSelThreads - 1 - tid;
            const uint32_t top = (key_top - 1u) >> kHistShift;
            const float per_item = 1400.f / (float)count_ge;              // aims at ~1500 buckets in all
            auto log2_buckets = [&](uint32_t h, uint32_t bin) -> int {    // -1: no bucket
                if (h == 0 || bin < b1 || bin > top) return -1;
                const float x = (float)h * per_item;
                return x <= 1.f ? 0 : min((int)(__log2f(x) + 0.5f), 11);
            };
            const int e0 = log2_buckets(h0, 2 * rt), e1 = log2_buckets(h1, 2 * rt + 1);
            const uint32_t nb0 = e0 < 0 ? 0u : 1u << e0, nb1 = e1 < 0 ? 0u : 1u << e1;
            const uint32_t incl = block_inclusive_scan<kSelThreads>(nb0 + nb1, sScan, &total);   // buckets of bins >= 2 rt
            adaptive = total != 0 && total <= (uint32_t)kBuckets;
            if (adaptive) {
                const uint32_t first0 = total - incl;                     // buckets of all lower bins
                if (e0 >= 0) sTab[2 * rt] = (uint16_t)(first0 | ((uint32_t)e0 << 11));
                if (e1 >= 0) sTab[2 * rt + 1] = (uint16_t)((first0 + nb0) | ((uint32_t)e1 << 11));
            }
            __syncthreads();
        }
        constexpr int kItems = kMaxCandidates / kSelThreads;
        uint64_t it[kItems];
        if (listed) {                                   // the dense list is in the workspace already
            const uint64_t* list = cand_list + bg * cand_cap;
#pragma unroll
            for (int u = 0; u < kItems; ++u) {
                const int e = u * kSelThreads + tid;
                it[u] = (e < (int)n_items) ? __hip_atomic_load(&list[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0ull;
            }
        } else {
#pragma unroll
            for (int u = 0; u < kItems; ++u) {
                const int e = u * kSelThreads + tid;
                it[u] = (e < (int)n_items) ? sKeys[e] : 0ull;
            }
        }
        const int n_mine = ((int)n_items - tid + kSelThreads - 1) / kSelThreads;   // items of this thread
        __syncthreads();                                // the list is in registers: sKeys is free
#pragma unroll
        for (int u = 0; u < kItems; ++u)
            if (u < n_mine) atomicAdd(&sCnt[bucket_of((uint32_t)(it[u] >> 32))], 0x10000u | item_len(it[u]));
        __syncthreads();
        // offsets from the top bucket down: thread 0 owns the two highest regular buckets
        const int rt = kSelThreads - 1 - tid;
        const uint32_t c0 = sCnt[2 * rt], c1 = sCnt[2 * rt + 1], cov = sCnt[kBuckets];
        const bool big = (c0 >> 16) > (uint32_t)kBucketLimit || (c1 >> 16) > (uint32_t)kBucketLimit ||
                         (cov >> 16) > (uint32_t)kBucketLimit;
        const uint32_t incl = block_inclusive_scan<kSelThreads>(c0 + c1, sScan, &total);
        const uint32_t above2 = incl - (c0 + c1) + cov;
        if (!__syncthreads_or(big ? 1 : 0)) {
            sStart[2 * rt + 1] = above2;      sCnt[2 * rt + 1] = above2 >> 16;
            sStart[2 * rt] = above2 + c1;     sCnt[2 * rt] = (above2 + c1) >> 16;
            if (tid == 0) { sStart[kBuckets] = 0; sCnt[kBuckets] = 0; }
            __syncthreads();
            // every item into its bucket (order inside a bucket is arbitrary)
#pragma unroll
            for (int u = 0; u < kItems; ++u)
                if (u < n_mine) sKeys[atomicAdd(&sCnt[bucket_of((uint32_t)(it[u] >> 32))], 1u)] = it[u];
            __syncthreads();
            // rank of a run's first position = positions in the buckets above + positions of the
            // larger runs in its own bucket; ranks below K' are the answer
            for (int e = tid; e < (int)n_items; e += kSelThreads) {
                const uint64_t item = sKeys[e];
                const uint32_t bk = bucket_of((uint32_t)(item >> 32));
                const uint32_t st = sStart[bk], lo = st >> 16, hi = sCnt[bk];
                uint32_t r = st & 0xFFFFu;
                // four reads in flight; a read past the bucket's end takes the item itself, which counts nothing
                for (uint32_t x = lo; x < hi; x += 4) {
                    uint64_t o[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) o[i] = sKeys[x + i < hi ? x + i : (uint32_t)e];
#pragma unroll
                    for (int i = 0; i < 4; ++i) r += (o[i] > item) ? item_len(o[i]) : 0u;
                }
                write_run(item, r);
            }
            for (int i = kprime + tid; i < k; i += kSelThreads) {
                idx[ob + i] = -1;
                if (sel_scores) sel_scores[ob + i] = 0.f;
            }
            return;
        }
        // a huge bucket (many equal or nearly equal scores): put the list back and sort it instead
#pragma unroll
        for (int u = 0; u < kItems; ++u)
            if (u < n_mine) sKeys[u * kSelThreads + tid] = it[u];
        nvalid = (int)n_items;
    } else {
        // ---- slow path: exact K-th largest image T by radix select over P ----
        // (bin b1 has been cut by the next 11 image bits above: 10 bits are left)
        __syncthreads();
        radix_pass<10>(P, n, prefix, mask, 0, kk, sHist, sScan, sOut);
        const uint32_t T = prefix | sOut[0];
        const uint32_t need_eq = kk - sOut[1];          // >= 1 positions with image == T are taken
        const uint32_t n_gt = (uint32_t)kprime - need_eq;
        __syncthreads();
        uint32_t base_eq = 0;
        for (int tile0 = 0; tile0 < n; tile0 += kSelThreads) {
            const int j = tile0 + tid;
            const bool in = j < n;
            const uint32_t key = in ? key_of(P[j]) : 0u;
            if (in && key > T) sKeys[atomicAdd(sCount, 1u)] = item_of(key, j);
            const bool eq = in && key == T;
            if (base_eq < need_eq) {                    // uniform over the workgroup
                if (__syncthreads_or(eq ? 1 : 0)) {
                    uint32_t total;
                    const uint32_t incl = block_inclusive_scan<kSelThreads>(eq ? 1u : 0u, sScan, &total);
                    const uint32_t rank = base_eq + incl - 1u;
                    if (eq && rank < need_eq) sKeys[n_gt + rank] = item_of(key, j);
                    base_eq += total;
                }
            }
        }
        nvalid = kprime;                                // runs of one position each
    }
    int npad = 1;
    while (npad < nvalid) npad <<= 1;
    for (int i = nvalid + tid; i < npad; i += kSelThreads) sKeys[i] = 0;   // sorts behind every real item
    __syncthreads();
    bitonic_sort_desc(sKeys, npad);
    // sKeys[0 .. nvalid) in order: a run's rank is the number of positions in the runs before it.
    // Every thread takes a stretch of the list: the lengths of the stretches before it, then its own.
    {
        const int per = (nvalid + kSelThreads - 1) / kSelThreads;
        const int e0 = min(tid * per, nvalid), e1 = min(e0 + per, nvalid);
        uint32_t mine = 0, total;
        for (int e = e0; e < e1; ++e) mine += item_len(sKeys[e]);
        uint32_t r = block_inclusive_scan<kSelThreads>(mine, sScan, &total) - mine;
        for (int e = e0; e < e1; ++e) {
            const uint64_t item = sKeys[e];
            write_run(item, r);
            r += item_len(item);
        }
    }
    for (int i = kprime + tid; i < k; i += kSelThreads) {
        idx[ob + i] = -1;
        if (sel_scores) sel_scores[ob + i] = 0.f;
    }
}

template <bool ADAPT>
__global__ __launch_bounds__(kSelThreads)
void select_kernel(const float* __restrict__ pooled, int64_t pooled_stride, const int32_t* seq_lens,
                   int32_t max_len, int32_t k, uint32_t* __restrict__ hist, int32_t cand_cap,
                   int32_t* __restrict__ idx, float* __restrict__ sel_scores,
                   const int32_t* pred, int32_t pred_val,
                   int32_t* __restrict__ sel_counters, uint64_t* __restrict__ cand_list) {
    select_body<ADAPT>(pooled, pooled_stride, seq_lens, max_len, k, hist, cand_cap, idx, sel_scores, pred, pred_val,
                       sel_counters, cand_list, (int)blockIdx.z, 1);
}

// The selections of several layers in one launch: grid z = layer * batch + sequence; what differs
// from layer to layer comes from a table passed by value.
struct SelectBatch {
    const float* pooled[kBatchLayers];
    uint32_t* hist[kBatchLayers];
    int32_t* idx[kBatchLayers];
    int32_t* sel_counters[kBatchLayers];
    uint64_t* cand_list[kBatchLayers];
    const int32_t* pred[kBatchLayers];       // NULL: every sequence of the layer
};

template <bool ADAPT>
__global__ __launch_bounds__(kSelThreads)
void select_batched_kernel(const SelectBatch tab, int32_t batch, int64_t pooled_stride, const int32_t* seq_lens,
                           int32_t max_len, int32_t k, int32_t cand_cap, int32_t pred_val, int32_t tile_vecs) {
    const int layer = blockIdx.z / batch, b = blockIdx.z - layer * batch;
    select_body<ADAPT>(tab.pooled[layer], pooled_stride, seq_lens, max_len, k, tab.hist[layer], cand_cap, tab.idx[layer],
                       nullptr, tab.pred[layer], pred_val, tab.sel_counters[layer], tab.cand_list[layer], b, tile_vecs);
}

}  // namespace rk

using namespace rk;

namespace rk {

int pool_stage(const rk_geom* geom, const float* weights, int64_t w_stride, const int32_t* seq_lens,
               int32_t max_len, int32_t pool_w, int32_t agg, const int32_t* pred, int32_t pred_val,
               const Workspace& ws, hipStream_t st) {
    const int G = geom->n_q_heads / geom->n_kv_heads;
    const int tile = pool_tile_for(max_len);
    dim3 pgrid((max_len + tile - 1) / tile, geom->n_kv_heads, geom->batch);
    if (tile == kPoolTileLong)
        hipLaunchKernelGGL((pool_hist_kernel<kPoolTileLong>), pgrid, dim3(256), 0, st, weights, w_stride, seq_lens, max_len,
                           geom->n_q_heads, geom->n_kv_heads, G, (pool_w - 1) / 2, agg, ws.pooled, pooled_row_stride(max_len), ws.hist,
                           pred, pred_val);
    else
        hipLaunchKernelGGL((pool_hist_kernel<kPoolTile>), pgrid, dim3(256), 0, st, weights, w_stride, seq_lens, max_len,
                           geom->n_q_heads, geom->n_kv_heads, G, (pool_w - 1) / 2, agg, ws.pooled, pooled_row_stride(max_len), ws.hist,
                           pred, pred_val);
    return launch_status();
}

int check_select_args(int32_t k, int32_t pool_w, int32_t agg, int32_t max_len) {
    if (pool_w < 1 || (pool_w & 1) == 0) return RK_ERR_INVALID_ARG;
    if (pool_w > RK_MAX_POOL_W || k > RK_MAX_K || agg < RK_AGG_MAX || agg > RK_AGG_FIRST) return RK_ERR_UNSUPPORTED;
    if ((int64_t)max_len > RK_MAX_SELECT_LEN) return RK_ERR_UNSUPPORTED;
    return RK_OK;
}

template <bool ADAPT>
static int launch_select(const rk_geom* geom, const int32_t* seq_lens, int32_t max_len, int32_t k, int32_t* idx,
                         float* sel_scores, const int32_t* pred, int32_t pred_val, const Workspace& ws, hipStream_t st) {
    // the sort kernel may need more than the default dynamic LDS; the per-bin bucket table is part
    // of it only where there can be kAdaptiveFrom candidates
    const size_t lds = (size_t)ws.cand_cap * sizeof(uint64_t) +
                       (2 * (kBuckets + 1) + kSelThreads / 64 + 4 + 1) * sizeof(uint32_t) +
                       (ADAPT ? kHistBins * sizeof(uint16_t) : 0);
    static size_t lds_allowed = 48 * 1024;       // grows monotonically (one per instantiation)
    if (lds > lds_allowed) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&select_kernel<ADAPT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return RK_ERR_UNSUPPORTED;
        }
        lds_allowed = lds;
    }
    // short rows: one workgroup per (sequence, KV head) does it all; longer ones: one per kSelTile positions
    const int tiles = max_len > kSelSingle ? (max_len + kSelTile - 1) / kSelTile : 1;
    dim3 sgrid(tiles, geom->n_kv_heads, geom->batch);
    hipLaunchKernelGGL((select_kernel<ADAPT>), sgrid, dim3(kSelThreads), lds, st, ws.pooled, pooled_row_stride(max_len), seq_lens,
                       max_len, k, ws.hist, ws.cand_cap, idx, sel_scores, pred, pred_val, ws.sel_counters, ws.cand_list);
    return launch_status();
}

template <bool ADAPT>
static int launch_select_batched(const rk_geom* geom, int n_layers, const Workspace* wss, int32_t* const* idx,
                                 const int32_t* seq_lens, int32_t max_len, int32_t k, const int32_t* const* pred,
                                 int32_t pred_val, hipStream_t st) {
    const int cand_cap = wss[0].cand_cap;
    const size_t lds = (size_t)cand_cap * sizeof(uint64_t) +
                       (2 * (kBuckets + 1) + kSelThreads / 64 + 4 + 1) * sizeof(uint32_t) +
                       (ADAPT ? kHistBins * sizeof(uint16_t) : 0);
    static size_t lds_allowed = 48 * 1024;
    if (lds > lds_allowed) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&select_batched_kernel<ADAPT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return RK_ERR_UNSUPPORTED;
        }
        lds_allowed = lds;
    }
    // Spreading a row over workgroups shortens one selection, but with many selections in one launch
    // the chip is full anyway and the hand-over between a row's workgroups only costs: measured at
    // 32k..128k rows, one workgroup per row wins from about 64 rows on (256 rows of 32k: 29 against 116 us).
    // Rows too long for one workgroup's registers (kSelHeld positions) are the exception: there a
    // workgroup per kSelHeld positions lists from registers what a single one would read in rounds.
    const int problems = (n_layers < kBatchLayers ? n_layers : kBatchLayers) * geom->batch * geom->n_kv_heads;
    int tiles = 1, tile_vecs = 1;
    if (max_len > kSelSingle && problems < kBatchSingleFrom) tiles = (max_len + kSelTile - 1) / kSelTile;
    else if (max_len >= 2 * kSelHeld) { tile_vecs = kSelHeld / kSelTile; tiles = (max_len + kSelHeld - 1) / kSelHeld; }
    for (int l0 = 0; l0 < n_layers; l0 += kBatchLayers) {
        const int n = n_layers - l0 < kBatchLayers ? n_layers - l0 : kBatchLayers;
        SelectBatch tab{};
        for (int l = 0; l < n; ++l) {
            const Workspace& w = wss[l0 + l];
            tab.pooled[l] = w.pooled; tab.hist[l] = w.hist; tab.idx[l] = idx[l0 + l];
            tab.sel_counters[l] = w.sel_counters; tab.cand_list[l] = w.cand_list;
            tab.pred[l] = pred ? pred[l0 + l] : nullptr;
        }
        dim3 grid(tiles, geom->n_kv_heads, n * geom->batch);
        hipLaunchKernelGGL((select_batched_kernel<ADAPT>), grid, dim3(kSelThreads), lds, st, tab, (int32_t)geom->batch,
                           pooled_row_stride(max_len), seq_lens, max_len, k, (int32_t)cand_cap, pred_val, (int32_t)tile_vecs);
        const int rc = launch_status();
        if (rc != RK_OK) return rc;
    }
    return RK_OK;
}

int select_batched_stage(const rk_geom* geom, int n_layers, const Workspace* wss, int32_t* const* idx,
                         const int32_t* seq_lens, int32_t max_len, int32_t k, const int32_t* const* pred, int32_t pred_val,
                         hipStream_t st) {
    if ((int64_t)kBatchLayers * geom->batch > 65535) return RK_ERR_UNSUPPORTED;      // grid z
    for (int l = 1; l < n_layers; ++l)
        if (wss[l].cand_cap != wss[0].cand_cap) return RK_ERR_INVALID_ARG;
    if (wss[0].cand_cap > kAdaptiveFrom) return launch_select_batched<true>(geom, n_layers, wss, idx, seq_lens, max_len, k, pred, pred_val, st);
    return launch_select_batched<false>(geom, n_layers, wss, idx, seq_lens, max_len, k, pred, pred_val, st);
}

// Two builds of the selection kernel: the one with the histogram-driven bucket layout serves the
// workspaces that can hold more than kAdaptiveFrom candidates (K > 4096); the other is the same
// code without it, because the smaller kernel measures faster where the layout is never used
// (1 us per layer of a full step at K = 2048 when it runs beside the attention kernel).
int select_stage(const rk_geom* geom, const int32_t* seq_lens, int32_t max_len, int32_t k, int32_t* idx,
                 float* sel_scores, const int32_t* pred, int32_t pred_val, const Workspace& ws, hipStream_t st) {
    if (ws.cand_cap > kAdaptiveFrom)
        return launch_select<true>(geom, seq_lens, max_len, k, idx, sel_scores, pred, pred_val, ws, st);
    return launch_select<false>(geom, seq_lens, max_len, k, idx, sel_scores, pred, pred_val, ws, st);
}

}  // namespace rk

extern "C" int rk_topk_select(const rk_geom* geom, const float* weights, int64_t w_stride,
                              const int32_t* seq_lens, int32_t max_len,
                              int32_t k, int32_t pool_w, int32_t agg,
                              int32_t* idx, float* sel_scores,
                              const int32_t* pred, int32_t pred_val,
                              void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!weights || !seq_lens || !idx || max_len <= 0 || k <= 0 || w_stride < max_len) return RK_ERR_INVALID_ARG;
    if ((rc = check_select_args(k, pool_w, agg, max_len)) != RK_OK) return rc;
    Workspace ws;
    if ((rc = check_workspace(geom, max_len, k, workspace, workspace_bytes, &ws)) != RK_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    if ((rc = pool_stage(geom, weights, w_stride, seq_lens, max_len, pool_w, agg, pred, pred_val, ws, st)) != RK_OK) return rc;
    return select_stage(geom, seq_lens, max_len, k, idx, sel_scores, pred, pred_val, ws, st);
}

extern "C" int rk_full_attn_select(const rk_geom* geom, const void* q, rk_kv full,
                                   const int32_t* seq_lens, int32_t max_len,
                                   void* out, float* weights, int64_t w_stride, float* lse,
                                   int32_t k, int32_t pool_w, int32_t agg,
                                   int32_t* idx, float* sel_scores,
                                   const int32_t* pred, int32_t pred_val,
                                   void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!q || !out || !seq_lens || !idx || max_len <= 0 || k <= 0) return RK_ERR_INVALID_ARG;
    if (!aligned16(q) || ((uintptr_t)out & 1u)) return RK_ERR_INVALID_ARG;
    if ((rc = check_kv(full)) != RK_OK) return rc;
    if (weights && (w_stride < max_len || ((uintptr_t)weights & 3u))) return RK_ERR_INVALID_ARG;
    if ((rc = check_select_args(k, pool_w, agg, max_len)) != RK_OK) return rc;
    Workspace ws;
    if ((rc = check_workspace(geom, max_len, k, workspace, workspace_bytes, &ws)) != RK_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    rc = full_attn_stage(geom, q, full, seq_lens, max_len, out, weights, w_stride, lse, pred, pred_val, ws, st,
                         false, (pool_w - 1) / 2, false, agg);
    if (rc != RK_OK) return rc;
    return select_stage(geom, seq_lens, max_len, k, idx, sel_scores, pred, pred_val, ws, st);
}

extern "C" int rk_score_select(const rk_geom* geom, const void* q, rk_kv full,
                               const int32_t* seq_lens, int32_t max_len,
                               float* weights, int64_t w_stride, float* lse,
                               int32_t k, int32_t pool_w, int32_t agg,
                               int32_t* idx, float* sel_scores,
                               const int32_t* pred, int32_t pred_val,
                               void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!q || !seq_lens || !idx || max_len <= 0 || k <= 0) return RK_ERR_INVALID_ARG;
    if (!aligned16(q)) return RK_ERR_INVALID_ARG;
    if ((rc = check_kv(full, false)) != RK_OK) return rc;
    if (weights && (w_stride < max_len || ((uintptr_t)weights & 3u))) return RK_ERR_INVALID_ARG;
    if ((rc = check_select_args(k, pool_w, agg, max_len)) != RK_OK) return rc;
    Workspace ws;
    if ((rc = check_workspace(geom, max_len, k, workspace, workspace_bytes, &ws)) != RK_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    rc = full_attn_stage(geom, q, full, seq_lens, max_len, nullptr, weights, w_stride, lse, pred, pred_val, ws, st,
                         false, (pool_w - 1) / 2, true, agg);
    if (rc != RK_OK) return rc;
    return select_stage(geom, seq_lens, max_len, k, idx, sel_scores, pred, pred_val, ws, st);
}

extern "C" int rk_full_attn_pool(const rk_geom* geom, const void* q, rk_kv full,
                                 const int32_t* seq_lens, int32_t max_len,
                                 void* out, float* weights, int64_t w_stride, float* lse,
                                 int32_t pool_w, int32_t agg, int32_t beside_other_work,
                                 const int32_t* pred, int32_t pred_val,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!q || !out || !seq_lens || max_len <= 0) return RK_ERR_INVALID_ARG;
    if (!aligned16(q) || ((uintptr_t)out & 1u)) return RK_ERR_INVALID_ARG;
    if ((rc = check_kv(full)) != RK_OK) return rc;
    if (weights && (w_stride < max_len || ((uintptr_t)weights & 3u))) return RK_ERR_INVALID_ARG;
    if ((rc = check_select_args(1, pool_w, agg, max_len)) != RK_OK) return rc;
    Workspace ws;
    if ((rc = check_workspace(geom, max_len, 0, workspace, workspace_bytes, &ws)) != RK_OK) return rc;
    return full_attn_stage(geom, q, full, seq_lens, max_len, out, weights, w_stride, lse, pred, pred_val, ws,
                           (hipStream_t)stream, false, (pool_w - 1) / 2, false, agg, beside_other_work != 0);
}

extern "C" int rk_full_attn_deferred(const rk_geom* geom, const void* q, rk_kv full,
                                     const int32_t* seq_lens, int32_t max_len, void* out, float* lse,
                                     const int32_t* pred, int32_t pred_val,
                                     void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!q || !out || !seq_lens || max_len <= 0) return RK_ERR_INVALID_ARG;
    if (!aligned16(q) || ((uintptr_t)out & 1u)) return RK_ERR_INVALID_ARG;
    if ((rc = check_kv(full)) != RK_OK) return rc;
    Workspace ws;
    if ((rc = check_workspace(geom, max_len, 0, workspace, workspace_bytes, &ws)) != RK_OK) return rc;
    return full_attn_stage(geom, q, full, seq_lens, max_len, out, nullptr, 0, lse, pred, pred_val, ws,
                           (hipStream_t)stream, false, 0, false, RK_AGG_MAX, false, true);
}

extern "C" int rk_select_pooled(const rk_geom* geom, const int32_t* seq_lens, int32_t max_len, int32_t k,
                                int32_t* idx, float* sel_scores, const int32_t* pred, int32_t pred_val,
                                void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!seq_lens || !idx || max_len <= 0 || k <= 0) return RK_ERR_INVALID_ARG;
    if ((rc = check_select_args(k, 1, RK_AGG_MAX, max_len)) != RK_OK) return rc;
    Workspace ws;
    if ((rc = check_workspace(geom, max_len, k, workspace, workspace_bytes, &ws)) != RK_OK) return rc;
    return select_stage(geom, seq_lens, max_len, k, idx, sel_scores, pred, pred_val, ws, (hipStream_t)stream);
}
