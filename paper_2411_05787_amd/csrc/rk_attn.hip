// Split-K decode attention for gfx950: rk_full_attn and rk_partial_attn.
//
// One workgroup reduces a chunk of KV rows of one (sequence, KV head) for all G query heads
// of the GQA group, so every K/V byte is read from HBM once.  The workgroup that arrives
// last for a (sequence, KV head) merges the partial results and writes the output.
//
// Hand-over between workgroups (which may sit on different XCDs, each with its own L2):
// partial results are written with agent-scope (write-through, coherent) stores and read with
// agent-scope loads.  No cache-wide release/acquire fence is used: on this chip one such fence
// per workgroup writes back and invalidates a whole L2 and costs more than the attention itself.
// Two forms (template parameter TAGGED):
//   tagged   every 16-byte row of a partial result carries the number of the call that wrote it.
//            A workgroup issues its rows and takes its arrival ticket at once, without waiting for
//            the rows to be acknowledged; the last arrival reads all rows and takes a row whose
//            tag is not this call's as still in flight: it reads that row again.  Every row it
//            waits for was issued before the ticket that made it the last arrival, so the wait
//            ends whatever else happens on the chip.
//   ticketed a writer waits until its stores are acknowledged (s_waitcnt vmcnt(0)) before it
//            takes its ticket; the last arrival can then rely on everything it reads.  One
//            round trip more; kept for scratch memory whose layout changes from call to call
//            (rk_partial_attn_static), where an old tag could sit where a new one is expected.
//
// Data path per wavefront and tile of 32 rows:
//   K rows  -> registers in MFMA operand layout (16-byte loads, no LDS)
//   S^T = K Q^T on the matrix cores: v_mfma_f32_16x16x32_bf16, M = 16 rows, N = query heads
//             (padded to 16), contraction over head_dim in 4 steps; a lane ends up with four
//             consecutive rows of one head
//   softmax bookkeeping (running max / sum per head) on those lanes; raw scores (when weights
//             are returned) are stored straight from them
//   O += P V on the matrix cores as well: P is already in operand layout (the contraction slots
//             of P V are numbered the way S^T left the rows in the lanes), split into two bf16
//             operands hi + lo so that it keeps ~17 bits; V rows are loaded with fully coalesced
//             16-byte loads, staged in LDS, and read back transposed (ds_read_b64_tr_b16) as the
//             other operand.  The fp32 O accumulators (8 tiles of 16 dims x 16 heads) do not
//             grow with the group size.
// The rows of a wavefront's next tile are requested as soon as the registers of the current tile
// are consumed (K after S^T, V after the copy to LDS), so loads are in flight during the rest of
// the tile's work.
#include "rk_internal.h"
#include "rk_device.h"

#include <atomic>
#include <mutex>

namespace rk {

struct AttnParams {
    const uint16_t* q;                 // bf16 [B, Hq, 128]
    const uint16_t* k1; const uint16_t* v1; int64_t s1_b, s1_h;   // small cache (TWO_SEG only)
    const uint16_t* k2; const uint16_t* v2; int64_t s2_b, s2_h;   // full cache
    const int32_t* tail_start;         // TWO_SEG only
    const int32_t* seq_lens;
    int32_t n_sel;                     // rows taken from the small cache (TWO_SEG only)
    int32_t evict;                     // ... less one per row decoded since the refresh (fixed-size small cache)
    int32_t tail_wg;                   // TWO_SEG: the rows of the full cache have a workgroup of their own (grid x = nch + 1)
    int32_t max_rows2;                 // host bound on the rows taken from the full cache
    int32_t cap1, cap2;                // rows allocated in the small / full cache
    int32_t nch;                       // workgroups per (sequence, KV head): the launch's grid x
    int32_t Hq, Hkv;
    float scale;
    uint16_t* out;                     // bf16 [B, Hq, 128]
    float* weights; int64_t w_stride;  // raw scores go here first (EMIT only)
    int32_t w_vec;                     // rows of `weights` start 16-byte aligned: vector stores allowed
    int32_t w_inter;                   // groups of 4 heads, scores kept in the workspace: the 4 heads of a position side by side
                                       // (score of head gi at position j of group (b, g): weights[(b*Hq + g*4) * w_stride + 4*j + gi])
    float* lse;                        // fp32 [B, Hq], never NULL here
    const int32_t* pred; int32_t pred_val;
    int32_t* counters; float* part_ml; float* part_o; int32_t max_chunks;
    uint32_t* epochs; uint32_t* tag_rows;     // TAGGED only: call number per (sequence, KV head), tagged partial results
    const int32_t* idx; int32_t idx_stride;   // LAZY only: the selection [B, Hkv, idx_stride] whose rows are not gathered yet
    float* trig_q_ref; float* trig_sim; int32_t* trig_need; float trig_threshold;   // TRIG only: the query-similarity test
    int32_t ragged_batch;              // != 0 (= batch): workgroups are shared out by length, see ragged_share_lane
    int32_t slice_merge;               // TAGGED: every workgroup merges a slice of the output (all workgroups of the launch are resident together)
    int32_t slice_spin;                // ... re-reading rows still in flight at most this often before it leaves its slice to the last one
};

// Work split of the split kernels.  The rows of a (sequence, KV head) are cut into tiles of 32;
// tile t belongs to wavefront t % 4 of workgroup (t / 4) % nch, so workgroup c starts at row
// 128 c and the tiles go round the nch * 4 wavefronts of the launch: every wavefront gets the
// same number of tiles, give or take one, whatever the length, and at any moment the launch
// streams one contiguous stretch of the cache.  Workgroups whose first row is past the end do
// nothing; the others each leave one partial result (the merge takes any subsets of the rows).
constexpr int kSplitWaves = 4, kTileRows = 32;
constexpr int kNoTailWg = 0xff;                   // top byte of the kernel argument s_b_and_tail: no workgroup for the tail rows
constexpr int kHeadsFirst = 0xfe;                 // ... (launches over the full cache only) grid x = KV head, y = sequence, z = chunk
__device__ __forceinline__ int active_workgroups(int n_rows, int nch) {
    return max(1, min(nch, (n_rows + kSplitWaves * kTileRows - 1) / (kSplitWaves * kTileRows)));
}

// Ragged batches.  With nch workgroups for every sequence, whatever its length, a launch that is
// resident as a whole takes as long as its longest sequence.  Score-emitting launches over
// 2..kRaggedMaxBatch sequences therefore share the nch * batch workgroups of a KV head out in
// proportion to the lengths: sequence i gets a_i = 1 + its share of the other nch * batch - batch by
// the largest-remainder rule (at least one, at most one per 128 rows and kMaxChunks; the a_i add up
// to no more than there are), and workgroup z * nch + x of the grid is number (that minus the a_j before it) of
// the sequence it falls into; those past the sum do nothing.  Every kernel of the call derives the
// same a_i from seq_lens: exact integer arithmetic, one wavefront, lane i for sequence i.
constexpr int kRaggedMaxBatch = 64;
__device__ __forceinline__ int clamped_len(int raw, int cap, int max_rows) { return min(max(min(raw, cap), 0), max_rows); }

// Lane i < batch: a_i.  Other lanes: 0.  Called by whole wavefronts.
__device__ __forceinline__ int ragged_share_lane(const int32_t* seq_lens, int batch, int nch, int cap, int max_rows) {
    const int lane = threadIdx.x & 63;
    const int len = lane < batch ? clamped_len(seq_lens[lane], cap, max_rows) : 0;
    long long total = len;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) total += __shfl_xor(total, d);
    const long long spare = (long long)nch * batch - batch;
    int a = 1;
    if (total > 0) {
        const long long num = spare * (long long)len;
        const long long fl = num / total;
        const long long rem = num - fl * total;
        // what the floors leave over goes, one each, to the largest remainders (ties: lower sequence first)
        long long given = fl;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) given += __shfl_xor(given, d);
        const int left = (int)(spare - given);                 // 0 <= left < batch
        int rank = 0;
        for (int j = 0; j < batch; ++j) {
            const long long rj = __shfl(rem, j);
            rank += (rj > rem || (rj == rem && j < lane)) ? 1 : 0;
        }
        a += (int)fl + (rank < left ? 1 : 0);
    }
    a = min(a, min(kMaxChunks, max(1, (len + kSplitWaves * kTileRows - 1) / (kSplitWaves * kTileRows))));
    return lane < batch ? a : 0;
}

// Partial results sequence b leaves behind (what active_workgroups is to the even split).
__device__ __forceinline__ int ragged_chunks_of(const AttnParams& p, int b) {
    const int a = ragged_share_lane(p.seq_lens, p.ragged_batch, p.nch, p.cap2, p.max_rows2);
    return __shfl(a, b);
}

// Sequence, number within it and share of the workgroup at `slot` (b < 0: none).
struct RaggedSlot { int b, c, nchunks; };
__device__ __forceinline__ RaggedSlot ragged_slot(const AttnParams& p, const int32_t* seq_lens, int slot) {
    const int lane = threadIdx.x & 63;
    const int a = ragged_share_lane(seq_lens, p.ragged_batch, p.nch, p.cap2, p.max_rows2);
    int incl = a;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d);
        if (lane >= d) incl += up;
    }
    const int before = incl - a;
    const unsigned long long hit = __ballot(a > 0 && before <= slot && slot < incl);
    RaggedSlot r{-1, 0, 0};
    if (hit != 0) {
        r.b = __ffsll(hit) - 1;
        r.c = slot - __shfl(before, r.b);
        r.nchunks = __shfl(a, r.b);
    }
    return r;
}

static inline int ragged_batch_of(const rk_geom* g) { return (g->batch > 1 && g->batch <= kRaggedMaxBatch) ? g->batch : 0; }

__device__ __forceinline__ void coherent_store2(float* p, float a, float b) {
    const uint64_t v = (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32);
    __hip_atomic_store(reinterpret_cast<uint64_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t coherent_load2(const float* p) {
    return __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float lo_f(uint64_t v) { return __uint_as_float((uint32_t)v); }
__device__ __forceinline__ float hi_f(uint64_t v) { return __uint_as_float((uint32_t)(v >> 32)); }
// All global stores this thread issued so far are acknowledged once this returns.
__device__ __forceinline__ void wait_stores_acknowledged() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Merge of the partial results of one (sequence, KV head); run by one whole workgroup.
//   M = max_c m_c;  L = sum_c e^{m_c - M} l_c;  out = sum_c e^{m_c - M} o_c / L;  lse = M + ln L
// Only one workgroup per (sequence, KV head) ever gets here, and nothing runs beside it on its
// CU: what it costs is the round trip of its loads plus one instruction after the other, so it is
// kept small (rolled loops, no fp64 library calls).  The partial outputs are read with 16-byte
// agent-scope loads, four consecutive dims of one chunk each (the read of kMergeBatch partial
// results of a group of 4 is 8 requests per thread; as 8-byte requests, 16 per thread, the same
// bytes took twice as long to come back), in batches of kMergeBatch chunks, two batches ahead of
// their use: up to 2 * kMergeBatch chunks cost one round trip, requested together with the
// (max, sum) pairs.  Where the outputs are fewer than half the threads, two halves of the
// workgroup take every other chunk and meet in LDS.
constexpr int kMergeBatch = 16;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

template <int G, int NW>
__device__ void merge_partials(const AttnParams& p, int b, int g, int nchunks, float* sW, float* sLc,
                               float* sM, double* sL) {
    constexpr int NT = NW * 64;
    constexpr int PER4 = G * kD / 4;              // groups of four consecutive dims to produce
    static_assert(PER4 <= NT, "one group of four dims per thread");
    constexpr int T = (2 * PER4 <= NT) ? 2 : 1;   // halves of the workgroup that share the chunks
    constexpr int LB = kMergeBatch / T;           // loads per thread and batch
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t bg = (int64_t)b * p.Hkv + g;
    const float* ml = p.part_ml + bg * kMaxChunks * G * 2;
    const float* po = p.part_o + bg * p.max_chunks * G * kD;
    const int n_ml = nchunks * G;
    static_assert(2 * NT >= kMergeChunks * RK_MAX_GROUP, "two loads per thread cover all (chunk, head) pairs");
    float* sRed = sLc + kMergeChunks * G;         // [PER4][4]: the second half's sums
    static_assert(NW * G * kD >= 2 * kMergeChunks * G + PER4 * 4, "merge scratch fits in the output staging buffer");

    const int half = tid / PER4, e4 = tid - half * PER4;          // (threads with half >= T only take part in the barriers)
    const bool active = half < T;
    const int gi = (4 * e4) / kD;
    // the partial outputs of this (sequence, KV head) as a buffer: reads past its end return 0
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(po), 0, (int)((int64_t)p.max_chunks * G * kD * sizeof(float)), 0x00020000);
    constexpr int kAgentScope = 16;               // cache-policy operand of the buffer load: sc1
    const int nb = (nchunks + kMergeBatch - 1) / kMergeBatch;
    u32x4_t cur[LB], nxt[LB];
    int r_batch = 0;                              // the next batch to request
    auto request = [&](u32x4_t (&dst)[LB]) {
        const int c0 = r_batch * kMergeBatch + (active ? half : 0);
#pragma unroll
        for (int u = 0; u < LB; ++u) {
            const int c = min(c0 + u * T, nchunks - 1);
            dst[u] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (c * G * kD + e4 * 4) * (int)sizeof(float), 0, kAgentScope);
        }
        ++r_batch;
    };
    // everything below is requested before the first wait
    const uint64_t ml0 = coherent_load2(ml + (int64_t)min(tid, n_ml - 1) * 2);
    const uint64_t ml1 = coherent_load2(ml + (int64_t)min(NT + tid, n_ml - 1) * 2);
    request(cur);
    if (nb > 1) request(nxt);
    if (tid < n_ml) { sW[tid] = lo_f(ml0); sLc[tid] = hi_f(ml0); }
    if (NT + tid < n_ml) { sW[NT + tid] = lo_f(ml1); sLc[NT + tid] = hi_f(ml1); }
    __syncthreads();
    // one wavefront per head: M = max_c m_c, w_c = e^{m_c - M} (overwrites m_c), L = sum_c w_c l_c
    for (int gj = w; gj < G; gj += NW) {
        const int c = min(lane, nchunks - 1);     // nchunks <= kMergeChunks = 64: one chunk per lane
        const float mc = sW[c * G + gj];
        const float mx = wave_max(mc);
        const float wgt = (lane >= nchunks || mc == -INFINITY) ? 0.f : fast_exp2((mc - mx) * kLog2e);
        double ls = (double)wgt * (double)sLc[c * G + gj];      // the sum that normalises the output: fp64
        if (lane < nb * kMergeBatch) sW[lane * G + gj] = wgt;    // zero beyond nchunks: whole batches are summed
        ls = wave_sum(ls);
        if (lane == 0) { sM[gj] = mx; sL[gj] = ls; }
    }
    __syncthreads();
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
    for (int batch = 0; batch < nb; ++batch) {
        const float* wrow = sW + (batch * kMergeBatch + (active ? half : 0)) * G + gi;
#pragma unroll
        for (int u = 0; u < LB; ++u) {
            const float wgt = wrow[u * T * G];
            acc[0] = fmaf(wgt, __uint_as_float(cur[u].x), acc[0]);
            acc[1] = fmaf(wgt, __uint_as_float(cur[u].y), acc[1]);
            acc[2] = fmaf(wgt, __uint_as_float(cur[u].z), acc[2]);
            acc[3] = fmaf(wgt, __uint_as_float(cur[u].w), acc[3]);
        }
#pragma unroll
        for (int u = 0; u < LB; ++u) cur[u] = nxt[u];
        if (batch + 2 < nb) request(nxt);
    }
    if (T == 2) {                                 // the second half hands its sums over
        if (half == 1) *reinterpret_cast<float4*>(sRed + e4 * 4) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        __syncthreads();
        if (half == 0) {
            const float4 o = *reinterpret_cast<const float4*>(sRed + e4 * 4);
            acc[0] += o.x; acc[1] += o.y; acc[2] += o.z; acc[3] += o.w;
        }
    }
    if (half == 0) {
        const float L = (float)sL[gi];
        const float inv = L > 0.f ? 1.f / L : 0.f;
        const uint2 packed = make_uint2((uint32_t)f32_to_bf16(acc[0] * inv) | ((uint32_t)f32_to_bf16(acc[1] * inv) << 16),
                                        (uint32_t)f32_to_bf16(acc[2] * inv) | ((uint32_t)f32_to_bf16(acc[3] * inv) << 16));
        reinterpret_cast<uint2*>(p.out + ((int64_t)b * p.Hq + g * G) * kD)[e4] = packed;
    }
    if (tid < G) {                                // fp32 log: lse is an fp32 output, M + ln L loses nothing that matters
        const float L = (float)sL[tid];
        p.lse[(int64_t)b * p.Hq + g * G + tid] = L > 0.f ? sM[tid] + logf(L) : -INFINITY;
    }
}

// ds_read_b64_tr_b16: every 16 lanes hand in 16 addresses of 4 consecutive bf16 (a 16 x 4
// matrix M, row = lane) and lane i gets back M[i/4 + 4e][i%4] for e = 0..3.
typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));      // 16 bytes in four registers
// 16-byte load of cache rows.  STREAM: the rows are read once per step and not again before
// far more than the caches hold has passed through (the full cache): a non-temporal load, which
// leaves the L2 and the last-level cache to the data that does come back (the small caches, read
// at every partial step).  Measured: the kernel that streams K and V of the full cache runs 4%
// faster with it; the partial step 3% slower and the K-only passes 3-5% slower, so only the
// former uses it.
template <bool STREAM>
__device__ __forceinline__ u32x4 load_rows16(const uint16_t* p) {
    if (STREAM) return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return *reinterpret_cast<const u32x4*>(p);
}
__device__ __forceinline__ v4s lds_read_tr16(const uint16_t* ptr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)ptr);
}
// Two fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// ---- tagged partial results ----
// The partial result of workgroup c of a (sequence, KV head) is G * 44 rows of 16 bytes.  For each
// head: 43 data rows { x[3r], x[3r+1], x[3r+2], tag } (the last holds two values) with
// x = (sum_j e^{s_j - m} v_j) / l the chunk's own normalised output, and one row
// { lambda, 0, 0, tag } with lambda = m + ln l, its log-sum-exp; tag is the number of the call.
// A row is one 16-byte store of one lane and one 16-byte load of one lane: it is never split, so
// a row whose tag is this call's holds this call's values.  The merge
//   Lambda = max_c lambda_c,  w_c = e^{lambda_c - Lambda},  out = sum_c w_c x_c / sum_c w_c
// needs no LDS and no barrier: the rows of a head are written by one wavefront of every workgroup
// (wavefront h % 4 for head h of the group) and merged by one wavefront of the workgroup that
// arrives last, lane r < 43 reading row r of every chunk and writing three elements.  lambda_c and
// the weights are the same for every lane: lane u takes chunk u's lambda, the wavefront reduces
// max and sum across lanes, and w_u reaches the other lanes as a scalar operand (v_readlane), which
// leaves three multiply-adds per chunk and lane.  Chunks are summed in order: the result does not
// depend on which workgroup merges or when.
constexpr int kTagSpinLimit = 1 << 16;            // re-reads of rows still in flight before giving up (NaN output)
constexpr int kAgentScopeAux = 16;                // cache-policy operand of buffer loads and stores: sc1

// (`rows`: the partial result of one workgroup, the same for all lanes; `row`: this lane's row of it)
__device__ __forceinline__ void store_tagged_row(uint32_t* rows, int n_rows, int row, float x0, float x1, float x2,
                                                 uint32_t tag) {
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(rows, 0, n_rows * 16, 0x00020000);
    const u32x4 v = {__float_as_uint(x0), __float_as_uint(x1), __float_as_uint(x2), tag};
    __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, row * 16, 0, kAgentScopeAux);
}

// Merge of the heads gi0, gi0 + 4, ... (NH of them; those >= G are skipped) of one (sequence, KV
// head) by one whole wavefront.  TB partial results per round trip: the loads of all NH heads are
// in flight together.
template <int G, int NH, int TB>
__device__ __forceinline__ void merge_tagged_heads(const AttnParams& p, int b, int g, int gi0, int nchunks_any_lane, uint32_t tag) {
    constexpr int ROWS = G * kTagRowsPerHead;
    static_assert(kTagDataRows <= 64 && TB <= 64, "one data row per lane, one chunk per lane");
    const int nchunks = __builtin_amdgcn_readfirstlane(nchunks_any_lane);      // the same in all lanes: kept in a scalar register
    const int lane = threadIdx.x & 63;
    const int64_t bg = (int64_t)b * p.Hkv + g;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        p.tag_rows + bg * kTagSlots * ROWS * 4, 0, kTagSlots * ROWS * 16, 0x00020000);
    const int r = min(lane, kTagDataRows - 1);
    float num[NH][3], den[NH], Lam[NH];
    bool good = true;
#pragma unroll
    for (int i = 0; i < NH; ++i) { num[i][0] = 0.f; num[i][1] = 0.f; num[i][2] = 0.f; den[i] = 0.f; Lam[i] = -INFINITY; }
#pragma unroll 1
    for (int c0 = 0; c0 < nchunks; c0 += TB) {                   // one round trip up to TB partial results
        u32x4 v[NH][TB], lt[NH];
        bool ok = false;
        int tries = 0;
        const int nb = min(nchunks - c0, TB);                    // partial results of this round (the same for all lanes)
        const int cl = c0 + min(lane, nb - 1);
        while (!__all(ok) && tries++ < kTagSpinLimit) {          // again only for rows that were still in flight
            if (tries > 1) __builtin_amdgcn_s_sleep(2);
#pragma unroll
            for (int i = 0; i < NH; ++i) {
                const int h0 = min(gi0 + i * kSplitWaves, G - 1) * kTagRowsPerHead;
                lt[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (cl * ROWS + h0 + kTagDataRows) * 16, 0, kAgentScopeAux);
#pragma unroll
                for (int u = 0; u < TB; ++u)
                    v[i][u] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, ((c0 + min(u, nb - 1)) * ROWS + h0 + r) * 16, 0, kAgentScopeAux);
            }
            ok = true;
#pragma unroll
            for (int i = 0; i < NH; ++i) {
                ok = ok && (lt[i].w == tag);
#pragma unroll
                for (int u = 0; u < TB; ++u) ok = ok && (v[i][u].w == tag);
            }
        }
        good = good && ok;
#pragma unroll
        for (int i = 0; i < NH; ++i) {
            const float lam = lane < nb ? __uint_as_float(lt[i].x) : -INFINITY;      // this lane's chunk, if it has one
            const float nl = fmaxf(fmaxf(Lam[i], wave_max(lam)), -3.0e38f);          // finite: exponents below are never inf - inf
            const float wv = fast_exp2((lam - nl) * kLog2e);                          // 0 for lanes without a chunk and for empty chunks
            const float so = fast_exp2((Lam[i] - nl) * kLog2e);
            float a0 = num[i][0] * so, a1 = num[i][1] * so, a2 = num[i][2] * so;
            den[i] = fmaf(den[i], so, wave_sum(wv));
#pragma unroll
            for (int u = 0; u < TB; ++u) {
                const float wu = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(wv), u));
                a0 = fmaf(wu, __uint_as_float(v[i][u].x), a0);
                a1 = fmaf(wu, __uint_as_float(v[i][u].y), a1);
                a2 = fmaf(wu, __uint_as_float(v[i][u].z), a2);
            }
            num[i][0] = a0; num[i][1] = a1; num[i][2] = a2; Lam[i] = nl;
        }
    }
#pragma unroll
    for (int i = 0; i < NH; ++i) {
        const int gi = gi0 + i * kSplitWaves;
        if (gi < G) {
            const float inv = den[i] > 0.f ? __builtin_amdgcn_rcpf(den[i]) : 0.f;
            const float nan = __uint_as_float(0x7fc00000u);
            const uint32_t p01 = good ? pack_bf16(num[i][0] * inv, num[i][1] * inv) : pack_bf16(nan, nan);
            const uint32_t p2 = good ? pack_bf16(num[i][2] * inv, 0.f) : pack_bf16(nan, 0.f);
            const int64_t bh = (int64_t)b * p.Hq + g * G + gi;
            uint16_t* o = p.out + bh * kD + 3 * lane;
            if (lane < kTagDataRows) {
                o[0] = (uint16_t)p01; o[1] = (uint16_t)(p01 >> 16);
                if (lane < kTagDataRows - 1) o[2] = (uint16_t)p2;
            }
            if (lane == 0) p.lse[bh] = den[i] > 0.f ? Lam[i] + __logf(den[i]) : -INFINITY;
        }
    }
}

// ---- merge by slices ----
// The same merge, shared out: workgroup c of the nchunks of a (sequence, KV head) merges a slice of its output,
// some consecutive data rows of one head (one per lane), reading them from every partial result.  One wavefront
// executes an instruction every 8 to 12 cycles however few lanes it uses (measured: 12 in a dependent chain), so
// the time of a merge is its instruction count, and this one is written for that: the offset of a chunk travels
// as the scalar operand of the loads, the slice is worked out long before (tag_slice_of, below), and the
// weights are taken against the first chunk's lambda, which every lane reads for itself, where that is safe
// (it saves the reduction for the maximum; any common reference gives the same quotient).  Whoever merges a
// slice: the same operations in the same order, the same bits.
struct TagSlice { int gi, r0, n_rows; };
// Which slice workgroup c merges: the workgroups c with c % G == gi share the 43 data rows of head gi
// (needs nchunks >= G: every head has a workgroup).
template <int G>
__device__ __forceinline__ TagSlice tag_slice_of(int c, int nchunks) {
    TagSlice s;
    s.gi = c % G;
    const int readers = (nchunks - s.gi + G - 1) / G;             // workgroups of this head
    const int per = (kTagDataRows + readers - 1) / readers;
    s.r0 = (c / G) * per;
    s.n_rows = min(per, kTagDataRows - s.r0);
    return s;
}

// TB: partial results read (at least nchunks).  Rows still in flight are re-read at most `spin` times; if
// some are still missing then, the output is left alone and the result is false (final: NaN is written instead).
template <int G, int TB>
__device__ __forceinline__ bool merge_tagged_slice(const AttnParams& p, int b, int g, const __amdgpu_buffer_rsrc_t rsrc, const TagSlice sl,
                                                   int nchunks, uint32_t tag, int spin, bool final) {
    constexpr int STRIDE = G * kTagRowsPerHead * 16;               // bytes of a partial result
    static_assert(TB <= 64, "one chunk per lane");
    const int lane = threadIdx.x & 63;
    const int r = sl.r0 + min(lane, sl.n_rows - 1);
    const int row_off = (sl.gi * kTagRowsPerHead + r) * 16;                                        // this lane's data row inside a partial result
    const int lam_off = min(lane, nchunks - 1) * STRIDE + (sl.gi * kTagRowsPerHead + kTagDataRows) * 16;   // lane u: chunk u's lambda row
    const int lam0_off = (sl.gi * kTagRowsPerHead + kTagDataRows) * 16;                            // the first chunk's, for every lane
    const int last = (nchunks - 1) * STRIDE;
    u32x4 v[TB], lt, l0;
    bool ok = false;
    int tries = 0;
    while (!__all(ok) && tries++ < spin) {
        if (tries > 1) __builtin_amdgcn_s_sleep(2);
        lt = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lam_off, 0, kAgentScopeAux);
        l0 = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lam0_off, 0, kAgentScopeAux);
#pragma unroll
        for (int u = 0; u < TB; ++u)
            v[u] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, row_off, min(u * STRIDE, last), kAgentScopeAux);
        uint32_t bad = (lt.w ^ tag) | (l0.w ^ tag);
#pragma unroll
        for (int u = 0; u < TB; ++u) bad |= v[u].w ^ tag;
        ok = bad == 0u;
    }
    const bool good = __all(ok);
    if (!good && !final) return false;
    const float lam = lane < nchunks ? __uint_as_float(lt.x) : -INFINITY;
    // reference: the first chunk's lambda, unless some chunk lies so far from it that a weight could overflow
    // or all could vanish (then the largest, by a reduction)
    float ref = __uint_as_float(l0.x);
    const bool near = lane >= nchunks || lam == -INFINITY || fabsf(lam - ref) < 20.f;
    if (!(ref > -3.0e38f) || !__all(near)) ref = fmaxf(wave_max(lam), -3.0e38f);
    const float wv = fast_exp2((lam - ref) * kLog2e);              // 0 for lanes without a chunk and for empty chunks
    const float den = wave_sum(wv);
    float a0 = 0.f, a1 = 0.f, a2 = 0.f;
#pragma unroll
    for (int u = 0; u < TB; ++u) {
        const float wu = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(wv), u));      // 0 beyond nchunks
        a0 = fmaf(wu, __uint_as_float(v[u].x), a0);
        a1 = fmaf(wu, __uint_as_float(v[u].y), a1);
        a2 = fmaf(wu, __uint_as_float(v[u].z), a2);
    }
    const float inv = den > 0.f ? __builtin_amdgcn_rcpf(den) : 0.f;
    const float nan = __uint_as_float(0x7fc00000u);
    const uint32_t p01 = good ? pack_bf16(a0 * inv, a1 * inv) : pack_bf16(nan, nan);
    const uint32_t p2 = good ? pack_bf16(a2 * inv, 0.f) : pack_bf16(nan, 0.f);
    const int64_t bh = (int64_t)b * p.Hq + g * G + sl.gi;
    uint16_t* o = p.out + bh * kD + 3 * r;
    if (lane < sl.n_rows) {
        o[0] = (uint16_t)p01; o[1] = (uint16_t)(p01 >> 16);
        if (r < kTagDataRows - 1) o[2] = (uint16_t)p2;
    }
    if (sl.r0 == 0) {                                              // (one slice per head)
        if (lane == 0) p.lse[bh] = good ? (den > 0.f ? ref + __logf(den) : -INFINITY) : nan;
    }
    return true;
}
// The same for slices of at most 16 rows, with four lanes to a row: lane 16 q + i sums the chunks q * per ..
// q * per + per - 1 (per = a quarter of the chunks, rounded up; TBP: at least that) for row r0 + i, and the four
// sums are added across the lanes, (q0 + q1) + (q2 + q3).  A lane's chunks are a quarter of the loads, checks and
// multiply-adds of the loop above; the weight of a chunk comes from the lane that holds it (ds_bpermute).
// Slots past the last chunk re-read the last chunk's row, with weight 0 (their weight lanes hold none).
template <int G, int TBP>
__device__ __forceinline__ bool merge_tagged_slice4(const AttnParams& p, int b, int g, const __amdgpu_buffer_rsrc_t rsrc, const TagSlice sl,
                                                    int nchunks, uint32_t tag, int spin, bool final) {
    constexpr int STRIDE = G * kTagRowsPerHead * 16;               // bytes of a partial result
    const int lane = threadIdx.x & 63;
    const int i = lane & 15, q = lane >> 4;
    const int per = (nchunks + 3) >> 2;
    const int r = sl.r0 + min(i, sl.n_rows - 1);
    const int row_off = (sl.gi * kTagRowsPerHead + r) * 16;
    const int lam_off = min(lane, nchunks - 1) * STRIDE + (sl.gi * kTagRowsPerHead + kTagDataRows) * 16;   // lane u: chunk u's lambda row
    const int lam0_off = (sl.gi * kTagRowsPerHead + kTagDataRows) * 16;                            // the first chunk's, for every lane
    const int first = q * per;                                     // this lane's first chunk
    const int base_v = row_off + first * STRIDE;
    const int limit_v = row_off + (nchunks - 1) * STRIDE;
    u32x4 v[TBP], lt, l0;
    bool ok = false;
    int tries = 0;
    while (!__all(ok) && tries++ < spin) {
        if (tries > 1) __builtin_amdgcn_s_sleep(2);
        lt = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lam_off, 0, kAgentScopeAux);
        l0 = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lam0_off, 0, kAgentScopeAux);
#pragma unroll
        for (int u = 0; u < TBP; ++u)
            v[u] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, min(base_v + u * STRIDE, limit_v), 0, kAgentScopeAux);
        uint32_t bad = (lt.w ^ tag) | (l0.w ^ tag);
#pragma unroll
        for (int u = 0; u < TBP; ++u) bad |= v[u].w ^ tag;
        ok = bad == 0u;
    }
    const bool good = __all(ok);
    if (!good && !final) return false;
    const float lam = lane < nchunks ? __uint_as_float(lt.x) : -INFINITY;
    float ref = __uint_as_float(l0.x);
    const bool near = lane >= nchunks || lam == -INFINITY || fabsf(lam - ref) < 20.f;
    if (!(ref > -3.0e38f) || !__all(near)) ref = fmaxf(wave_max(lam), -3.0e38f);
    const float wv = fast_exp2((lam - ref) * kLog2e);              // 0 for lanes without a chunk and for empty chunks
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, den = 0.f;
#pragma unroll
    for (int u = 0; u < TBP; ++u) {
        // (slot u of quarter q is chunk first + u; for u >= per it belongs to the next quarter: weight 0)
        const float wu = __int_as_float(__builtin_amdgcn_ds_bpermute((first + u) * 4, __float_as_int(wv)));
        const float wq = u < per ? wu : 0.f;
        a0 = fmaf(wq, __uint_as_float(v[u].x), a0);
        a1 = fmaf(wq, __uint_as_float(v[u].y), a1);
        a2 = fmaf(wq, __uint_as_float(v[u].z), a2);
        den += wq;
    }
    a0 = sum_xor32(sum_xor16(a0)); a1 = sum_xor32(sum_xor16(a1)); a2 = sum_xor32(sum_xor16(a2)); den = sum_xor32(sum_xor16(den));
    const float inv = den > 0.f ? __builtin_amdgcn_rcpf(den) : 0.f;
    const float nan = __uint_as_float(0x7fc00000u);
    const uint32_t p01 = good ? pack_bf16(a0 * inv, a1 * inv) : pack_bf16(nan, nan);
    const uint32_t p2 = good ? pack_bf16(a2 * inv, 0.f) : pack_bf16(nan, 0.f);
    const int64_t bh = (int64_t)b * p.Hq + g * G + sl.gi;
    uint16_t* o = p.out + bh * kD + 3 * r;
    if (lane < sl.n_rows) {
        o[0] = (uint16_t)p01; o[1] = (uint16_t)(p01 >> 16);
        if (r < kTagDataRows - 1) o[2] = (uint16_t)p2;
    }
    if (sl.r0 == 0) {                                              // (one slice per head)
        if (lane == 0) p.lse[bh] = good ? (den > 0.f ? ref + __logf(den) : -INFINITY) : nan;
    }
    return true;
}
// (17 partial results at the shape that matters most: 16 workgroups for 2048 selected rows and one for the
// rows decoded since; otherwise up to 20)
template <int G>
__device__ __forceinline__ bool merge_tagged_slice_n(const AttnParams& p, int b, int g, const __amdgpu_buffer_rsrc_t rsrc, const TagSlice sl,
                                                     int nchunks, uint32_t tag, int spin, bool final) {
    if (sl.n_rows <= 16 && nchunks > 4) {
        if (nchunks <= 20) return merge_tagged_slice4<G, 5>(p, b, g, rsrc, sl, nchunks, tag, spin, final);
        if (nchunks <= 36) return merge_tagged_slice4<G, 9>(p, b, g, rsrc, sl, nchunks, tag, spin, final);
        return merge_tagged_slice4<G, 16>(p, b, g, rsrc, sl, nchunks, tag, spin, final);
    }
    if (nchunks <= 17) return merge_tagged_slice<G, 17>(p, b, g, rsrc, sl, nchunks, tag, spin, final);
    return merge_tagged_slice<G, 20>(p, b, g, rsrc, sl, nchunks, tag, spin, final);
}
constexpr int kSliceChunks = 20, kSliceChunks4 = 64;   // the merge by slices serves up to this many partial results (slices of up to 16 rows: the latter)

// Roles of lane (n16, c4) = (lane % 16, lane / 16) of a wavefront, per tile of 32 rows:
//   K operand   row n16 of a 16-row half tile, dims 8*(4*kk + c4) .. +7, kk = 0..3
//   Q operand   head n16 (zero beyond G), same dims
//   S^T result  head n16, rows 4*c4 + i (i = 0..3) of each half tile
//   V load      rows c4 + 4*jj (jj = 0..7), dims 8*n16 .. +7
//   P operand   head n16, contraction slot e = 4*t + i  <->  row 16*t + 4*c4 + i
//   V operand   dim 16*dt + n16, the same slots (LDS transpose read)
//   O result    dim 16*dt + n16, heads 4*c4 + i
#ifndef RK_EMIT_OCCUPANCY
#define RK_EMIT_OCCUPANCY 3       // workgroups per CU the score-emitting kernel is compiled for
#endif
// LAZY (with TWO_SEG): the first partial step after a refresh whose gather was left out.  The rows
// of the small-cache segment are read from the full cache through the selection (row r of the list
// is row idx[r] of the full cache) and written to the small cache on the way, so that the step
// leaves the small cache as rk_gather_small_kv would have.  k_first / v_first / s_b / s_h then
// describe the FULL cache and `pred` carries the selection (the predicate is read from `p`).

// TRIG (with TWO_SEG): the partial step of a step on which the query-similarity trigger is tested
// (Section 2.2).  Every workgroup works the test out for itself from the 9 KB of queries and
// reference, behind the requests for its first tile and before it waits for anything, and gives up
// if its sequence needs a full step: the test costs no launch of its own and no launch waits for it.
// Workgroup (0, 0) of the sequence stores the similarity and the decision for the launches that
// follow (the full step under that predicate).  Where the test asks for a full step the averaged
// query becomes the new reference; every workgroup of the sequence has read the old one by then:
// each takes a ticket after its test, and the last one stores.
template <int G, int NW, bool EMIT, bool TWO_SEG, bool LAZY = false, bool TAGGED = !EMIT, bool TRIG = false>
__global__ __launch_bounds__(NW * 64, (EMIT && !TAGGED) ? RK_EMIT_OCCUPANCY : 2)
void attn_split_kernel(const uint16_t* k_first, const uint16_t* v_first, int64_t s_b_and_tail, int32_t s_h, int32_t spec_rows,
                       const int32_t* seq_lens, const int32_t* tail_start, const int32_t* pred, const uint32_t* epochs,
                       const AttnParams p) {
    static_assert(!LAZY || (TWO_SEG && !EMIT), "the lazy gather belongs to the partial step");
    // (EMIT with TAGGED: the scores go out as usual, and the output is merged inside the kernel all the same; the
    // per-chunk (max, sum) pairs are still stored for the kernels that turn the scores into weights)
    static_assert(!TRIG || (TWO_SEG && !LAZY), "the trigger is tested by the partial step");
    // The leading arguments repeat what the first loads need (the cache that holds the first rows,
    // its strides, the two length arrays, the predicate, the call numbers): 16 dwords that the command processor
    // hands over in registers at wavefront launch (kernel-argument preload), so neither the first
    // K/V request nor the read of the lengths waits for a read of the argument block.  Everything
    // else comes from `p` as before (tail_start is NULL unless TWO_SEG).  A launch with a predicate
    // does wait for it (and for p.pred_val) before it requests anything: a switched-off sequence
    // must not cost memory traffic.
    constexpr int ROWS = kTileRows;          // rows per wavefront and tile = contraction depth of P V
    static_assert(NW == kSplitWaves, "work split");
    constexpr int NV = ROWS / 4;             // V loads per lane and tile
    constexpr int NC = (G + 3) / 4;          // lane groups whose O accumulators hold real heads
    constexpr int NT = NW * 64;
    constexpr int VS = kD + 8;               // LDS row stride of the V tile (272 bytes: rows spread over banks)

    // The sequence stride also carries, in its top byte, the grid x of the workgroup that takes the
    // rows of the full cache on its own (kNoTailWg: none; see tail_mode below): like everything the
    // first loads need, it is there when the wavefront starts.
    const int64_t s_b = s_b_and_tail & ((1ll << 56) - 1);
    const int tail_c = (int)(s_b_and_tail >> 56) & 0xff;
    // kHeadsFirst in the same byte (launches of the full-cache kernel over one sequence or an evenly split
    // batch): the KV head is grid x and the chunk grid z.  Workgroups are handed out in the grid's linear
    // order, x fastest, and go to the 8 XCDs in turn: with the heads as x every XCD streams the same
    // KV heads from start to end instead of every eighth chunk of all heads.
    const bool heads_first = !TWO_SEG && tail_c == kHeadsFirst;
    int c = heads_first ? blockIdx.z : blockIdx.x, b = heads_first ? blockIdx.y : blockIdx.z, nch_b = p.nch;
    const int g = heads_first ? blockIdx.x : blockIdx.y;
    const int n_kv = heads_first ? gridDim.x : gridDim.y;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n16 = lane & 15, c4 = lane >> 4;
    constexpr bool kCanBeRagged = EMIT && !TWO_SEG;
    if (kCanBeRagged && p.ragged_batch != 0) {           // which sequence this workgroup works for: by length
        const RaggedSlot rs = ragged_slot(p, seq_lens, (int)(blockIdx.z * p.nch + blockIdx.x));
        if (rs.b < 0) return;
        b = __builtin_amdgcn_readfirstlane(rs.b);
        c = __builtin_amdgcn_readfirstlane(rs.c);
        nch_b = __builtin_amdgcn_readfirstlane(rs.nchunks);
    }
    // LAZY: the selection's entries for the rows of a tile, lane i < 32 holding that of row r + i
    // (clamped into the full cache: a bad index reads a wrong row, never outside the cache)
    const int32_t* sel = LAZY ? pred + ((int64_t)b * n_kv + g) * spec_rows : nullptr;   // idx_stride == spec_rows
    auto tile_sel = [&](int r, int n_rows) -> int {
        const int j = min(r + (lane & 31), n_rows - 1);
        return LAZY ? sel[max(j, 0)] : 0;
    };
    int sel0 = 0;
    if (LAZY) {
        sel0 = tile_sel((c * NW + w) * kTileRows, spec_rows);      // before anything else: the rows depend on it
        if (p.pred != nullptr && p.pred[b] != p.pred_val) return;
    } else {
        if (!TRIG && pred != nullptr && pred[b] != p.pred_val) return;
    }

    // TRIG: the test's queries and reference are requested first of all, so that the test is worked out
    // while the first tile is on its way (memory answers in the order of the requests).  A launch with
    // the test has no predicate, and takes the call numbers from the argument block: the two
    // preloaded pointers carry the queries and the reference instead.
    // One wavefront of the workgroup does it (all the workgroups of the launch read the same 9 KB at
    // the same time: four times the requests cost more than the barrier that passes the result on).
    SimLoads trig_ld;
    if constexpr (TRIG) {
        if (w == 0)
            similarity_request(reinterpret_cast<const uint16_t*>(pred), reinterpret_cast<const float*>(epochs), b, n_kv * G, trig_ld);
    }

    // ---- K and V rows of the first tile are requested before any length is known ----
    // Rows below `spec_rows` exist whatever the device-side lengths say (small cache: the first
    // n_sel rows; full cache: its capacity), so a workgroup whose first 128 rows lie wholly below
    // it may read them at once; rows that turn out to be past the end are masked like any other.
    // This takes the round trip for seq_lens / tail_start off the critical path.
    // TWO_SEG with p.tail_wg: the launch has one workgroup more per (sequence, KV head), the last of
    // grid x, which takes the rows of the full cache (the tokens decoded since the refresh) and
    // nothing else; the others share the rows of the small cache.  Those few rows then cost no
    // wavefront a second tile: the workgroup that has them finishes with the others, not a tile later.
    const bool tail_mode = TWO_SEG && !LAZY && tail_c != kNoTailWg && tail_c != kHeadsFirst;
    const bool is_tail = tail_mode && c == tail_c;
    int r_first = (c * NW + w) * ROWS;
    const bool spec = !is_tail && (c + 1) * NW * ROWS <= spec_rows;     // spec_rows: min(n_sel, cap1) or cap2
    u32x4 kA[2][4], vA[NV];
    if (spec) {
        const uint16_t* kspec = k_first + (int64_t)b * s_b + (int64_t)g * s_h + c4 * 8;
        const int cap_full = p.cap2;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int64_t row = LAZY ? min(max(__shfl(sel0, t * 16 + n16), 0), cap_full - 1) : r_first + t * 16 + n16;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                kA[t][kk] = load_rows16<!TWO_SEG>(kspec + row * kD + kk * 32);
        }
        const uint16_t* vspec = v_first + (int64_t)b * s_b + (int64_t)g * s_h + n16 * 8;
#pragma unroll
        for (int jj = 0; jj < NV; ++jj) {
            const int64_t row = LAZY ? min(max(__shfl(sel0, jj * 4 + c4), 0), cap_full - 1) : r_first + jj * 4 + c4;
            vA[jj] = load_rows16<!TWO_SEG>(vspec + row * kD);
        }
    }

    // ---- Q (head n16, dims 8*(4*kk + c4) .. +7) and the two lengths ----
    // Requested here, behind the first tile and before anything waits: left to itself the compiler
    // moves the Q loads down to their first use, below the branch that needs the lengths, and
    // puts a wait between the two length loads, so that Q arrived a round trip after the lengths
    // and the lengths one after the other (8.42 -> 8.24 us per partial step).  The
    // condition is always true; it only keeps the requests in a block of their own, up here.
    bf16x8 qa[4];
    int len_raw = 0, tail_raw = 0;
    constexpr int UPW = (G + NW - 1) / NW;    // TAGGED: heads whose rows this wavefront publishes and merges (heads w, w + NW)
    uint32_t epoch = 0;                       // ... and the number of the last call that merged this (sequence, KV head)
    {
        uint4 qu[4] = {make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0)};
        if (spec_rows >= 0) {
            len_raw = seq_lens[b];
            if (TWO_SEG) tail_raw = tail_start[b];
            if (TAGGED) epoch = (TRIG ? p.epochs : epochs)[(int64_t)b * n_kv + g];
            const uint16_t* qrow = p.q + ((int64_t)b * p.Hq + (int64_t)g * G + (n16 < G ? n16 : 0)) * kD;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) qu[kk] = *reinterpret_cast<const uint4*>(qrow + (kk * 4 + c4) * 8);
        }
        // TRIG: the test is worked out here, between the requests and the first wait for a tile
        if constexpr (TRIG) {
            __shared__ int trig_last, trig_need_full;
            float qbar[8];
            if (w == 0) {
                const float s = similarity_finish(reinterpret_cast<const uint16_t*>(pred), b, n_kv * G, trig_ld, qbar);
                const bool need_w = !(s > p.trig_threshold);
                if (lane == 0) {
                    trig_need_full = need_w ? 1 : 0;
                    if (c == 0 && g == 0) { p.trig_sim[b] = s; p.trig_need[b] = need_w ? 1 : 0; }
                }
            }
            __syncthreads();
            const bool need = trig_need_full != 0;
            if (need) {
                // (the ticket is the second word of the sequence's first arrival-counter line: zero between launches;
                // the wavefront that takes it is the one that read the reference)
                if (tid == 0) {
                    int32_t* ticket = p.counters + (int64_t)b * n_kv * kCounterStride + 1;
                    const int seen = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    trig_last = seen == (int)(gridDim.x * gridDim.y) - 1 ? 1 : 0;
                    if (trig_last) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                __syncthreads();
                if (trig_last && tid < 16) {
                    float4* rp = reinterpret_cast<float4*>(p.trig_q_ref + (int64_t)b * kD + tid * 8);
                    rp[0] = make_float4(qbar[0], qbar[1], qbar[2], qbar[3]);
                    rp[1] = make_float4(qbar[4], qbar[5], qbar[6], qbar[7]);
                }
                return;
            }
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (n16 >= G) qu[kk] = make_uint4(0, 0, 0, 0);
            qa[kk] = __builtin_bit_cast(bf16x8, qu[kk]);
        }
    }

    // ---- the row list of this (sequence, KV head) ----
    // (device-side lengths are clamped to the allocated rows: no access leaves the caches)
    const int len = min(len_raw, p.cap2);
    int n1 = 0, start2 = 0;
    if (TWO_SEG) {
        const int t0 = min(max(tail_raw, 0), p.cap2);
        // fixed-size small cache: every row decoded since the refresh pushed out the selected row
        // with the lowest score, i.e. the last one (the small cache is in descending score order)
        const int keep = p.evict ? max(p.n_sel - max(len - t0, 0), 0) : p.n_sel;
        n1 = min(min(keep, t0), p.cap1);
        n1 = max(n1, 0);
        start2 = t0;
    }
    const int n2 = min(max(len - start2, 0), p.max_rows2);
    const int n = n1 + n2;
    int nchunks, row1 = n, c_rec = c, n_split;          // partial results in all; end of this workgroup's rows; its slot; workgroups it shares rows with
    if (tail_mode) {
        const int n_main = (n1 > 0 || n2 == 0) ? active_workgroups(n1, p.nch) : 0;
        nchunks = n_main + (n2 > 0 ? 1 : 0);
        if (is_tail) {
            if (n2 == 0) return;
            c_rec = n_main; r_first = n1 + w * ROWS; n_split = 1;
        } else {
            if (c >= n_main) return;
            row1 = n1; n_split = n_main;
        }
    } else {
        nchunks = (kCanBeRagged && p.ragged_batch != 0) ? nch_b : active_workgroups(n, p.nch);
        if (c >= nchunks) return;
        n_split = nchunks;
    }

    const uint16_t* kb1 = nullptr; const uint16_t* vb1 = nullptr;
    if (TWO_SEG) {
        kb1 = p.k1 + (int64_t)b * p.s1_b + (int64_t)g * p.s1_h;
        vb1 = p.v1 + (int64_t)b * p.s1_b + (int64_t)g * p.s1_h;
    }
    // row r of the list lives at base2 + (start2 + r - n1) * 128 once r >= n1
    const uint16_t* kb2 = p.k2 + (int64_t)b * p.s2_b + (int64_t)g * p.s2_h + (int64_t)(start2 - n1) * kD;
    const uint16_t* vb2 = p.v2 + (int64_t)b * p.s2_b + (int64_t)g * p.s2_h + (int64_t)(start2 - n1) * kD;

    // TAGGED: this workgroup's share of the merge by slices (see there), worked out here, while the first tile is
    // on its way, and not between publishing and merging
    TagSlice my_slice = {0, 0, 0};
    bool slices_fit = false;                  // every head has a workgroup, and the merge has a form for this many partial results
    __amdgpu_buffer_rsrc_t tag_rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)nullptr, 0, 0, 0x00020000);
    if (TAGGED) {
        if (nchunks >= G) {
            my_slice = tag_slice_of<G>(c_rec, nchunks);
            const int fewest = nchunks / G;                        // workgroups of the head that has fewest: the longest slices
            slices_fit = nchunks <= kSliceChunks || (nchunks <= kSliceChunks4 && (kTagDataRows + fewest - 1) / fewest <= 16);
        }
        my_slice.gi = __builtin_amdgcn_readfirstlane(my_slice.gi);
        my_slice.r0 = __builtin_amdgcn_readfirstlane(my_slice.r0);
        my_slice.n_rows = __builtin_amdgcn_readfirstlane(my_slice.n_rows);
        tag_rsrc = __builtin_amdgcn_make_buffer_rsrc(p.tag_rows + ((int64_t)b * p.Hkv + g) * kTagSlots * (G * kTagRowsPerHead) * 4, 0,
                                                     kTagSlots * G * kTagRowsPerHead * 16, 0x00020000);
    }

    __shared__ __attribute__((aligned(16))) uint16_t sV[NW][ROWS][VS];
    __shared__ __attribute__((aligned(16))) float sAlpha[NW][16];
    __shared__ __attribute__((aligned(16))) float sMw[NW][16];
    __shared__ __attribute__((aligned(16))) float sLw[NW][16];
    __shared__ __attribute__((aligned(16))) float sO[NW][G][kD];       // reused by the merge
    __shared__ float sMf[8];
    __shared__ double sLf[8];
    __shared__ int sTicket;
    static_assert(NW * G * kD >= 2 * kMergeChunks * G + G * kD, "merge scratch must fit in the output staging buffer");

    float m_run = -INFINITY, l_run = 0.f;          // of head n16, over the rows this lane group saw
    f32x4 acc_o[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) acc_o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // ---- loads: rows past the end of the chunk re-read its last row (masked later) ----
    // (LAZY: kfull / vfull are row 0 of the full cache of this (sequence, KV head))
    const uint16_t* kfull = LAZY ? p.k2 + (int64_t)b * p.s2_b + (int64_t)g * p.s2_h : nullptr;
    const uint16_t* vfull = LAZY ? p.v2 + (int64_t)b * p.s2_b + (int64_t)g * p.s2_h : nullptr;
    auto load_k = [&](int r) {
        const int sv = LAZY ? tile_sel(r, n1) : 0;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int row = min(r + t * 16 + n16, row1 - 1);
            const int srow = LAZY ? __shfl(sv, t * 16 + n16) : 0;       // (all lanes take part)
            const uint16_t* rp;
            if (LAZY && row < n1) {
                rp = kfull + (int64_t)min(max(srow, 0), p.cap2 - 1) * kD + c4 * 8;
            } else {
                const uint16_t* base = (TWO_SEG && row < n1) ? kb1 : kb2;
                rp = base + (int64_t)row * kD + c4 * 8;
            }
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) kA[t][kk] = load_rows16<!TWO_SEG>(rp + kk * 32);
        }
    };
    auto load_v = [&](int r) {
        const int sv = LAZY ? tile_sel(r, n1) : 0;
#pragma unroll
        for (int jj = 0; jj < NV; ++jj) {
            const int row = min(r + jj * 4 + c4, row1 - 1);
            const int srow = LAZY ? __shfl(sv, jj * 4 + c4) : 0;
            if (LAZY && row < n1) {
                vA[jj] = load_rows16<!TWO_SEG>(vfull + (int64_t)min(max(srow, 0), p.cap2 - 1) * kD + n16 * 8);
            } else {
                const uint16_t* base = (TWO_SEG && row < n1) ? vb1 : vb2;
                vA[jj] = load_rows16<!TWO_SEG>(base + (int64_t)row * kD + n16 * 8);
            }
        }
    };
    // One tile.  The K registers are free again once S^T is computed and the V registers once the
    // tile sits in LDS: the next tile's rows are requested at those two points, so its loads are
    // in flight during the rest of this tile's work.
    auto compute_tile = [&](int r, int r_next) -> int {
        if (LAZY) {       // the K rows of the selection go to their slots of the small cache (bit copies)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int row = r + t * 16 + n16;
                if (row < n1) {
                    uint16_t* dst = const_cast<uint16_t*>(kb1) + (int64_t)row * kD + c4 * 8;
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) *reinterpret_cast<u32x4*>(dst + kk * 32) = kA[t][kk];
                }
            }
        }
        // ---- S^T = K Q^T on the matrix cores: head n16, rows r + 16 t + 4 c4 + i ----
        float s[2][4];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kA[t][kk]), qa[kk], acc, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 4; ++i) s[t][i] = (r + t * 16 + 4 * c4 + i < row1) ? acc[i] * p.scale : -INFINITY;
        }
        if (r_next < row1) load_k(r_next);
        // ---- raw scores out: four consecutive rows of one head per lane, one 16-byte store
        //      where the row of the weights tensor allows it ----
        if (EMIT && G == 4 && p.w_inter) {
            // The scores of a position's four heads as one 16-byte record: a tile of 32 rows leaves as
            // one contiguous stretch of 512 bytes instead of four stretches of 128 bytes 4 * w_stride
            // bytes apart (measured on the kernel alone: 107.4 -> 102.8 us per launch at 131072 rows,
            // 26.6 -> 26.3 at 32768).  The lanes n16 = 0..3 of a row of 16 hold heads 0..3 for rows
            // first .. first + 3: a 4 x 4 transpose inside the quad (two exchange steps on the DPP
            // operand path) gives lane h the four heads of row first + h.  All lanes take part.
            float* blk = p.weights + ((int64_t)b * p.Hq + (int64_t)g * G) * p.w_stride;
            const bool odd1 = (n16 & 1) != 0, odd2 = (n16 & 2) != 0;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                float a0 = s[t][0], a1 = s[t][1], a2 = s[t][2], a3 = s[t][3];
                const float y01 = dpp_move_f<kDppXor1>(odd1 ? a0 : a1), y23 = dpp_move_f<kDppXor1>(odd1 ? a2 : a3);
                a0 = odd1 ? y01 : a0; a1 = odd1 ? a1 : y01; a2 = odd1 ? y23 : a2; a3 = odd1 ? a3 : y23;
                const float z02 = dpp_move_f<kDppXor2>(odd2 ? a0 : a2), z13 = dpp_move_f<kDppXor2>(odd2 ? a1 : a3);
                a0 = odd2 ? z02 : a0; a2 = odd2 ? a2 : z02; a1 = odd2 ? z13 : a1; a3 = odd2 ? a3 : z13;
                const int row = r + t * 16 + 4 * c4 + (n16 & 3);
                if (n16 < 4 && row < row1) *reinterpret_cast<float4*>(blk + (int64_t)row * 4) = make_float4(a0, a1, a2, a3);
            }
        } else if (EMIT && p.weights != nullptr) {
            if (n16 < G) {
                float* wrow = p.weights + ((int64_t)b * p.Hq + (int64_t)g * G + n16) * p.w_stride + r + 4 * c4;
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int first = r + t * 16 + 4 * c4;
                    if (p.w_vec && first + 4 <= row1) {
                        *reinterpret_cast<float4*>(wrow + t * 16) = make_float4(s[t][0], s[t][1], s[t][2], s[t][3]);
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (first + i < row1) wrow[t * 16 + i] = s[t][i];
                    }
                }
            }
        }
        // ---- running softmax statistics of head n16 (row r itself is always valid: finite max) ----
        float mx = fmaxf(fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3])),
                         fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3])));
        mx = max_xor32(max_xor16(mx));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = fast_exp2((m_run - m_new) * kLog2e);
        m_run = m_new;
        float pr[8], ps = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            pr[e] = fast_exp2((s[e >> 2][e & 3] - m_new) * kLog2e);
            ps += pr[e];
        }
        l_run = l_run * alpha + ps;                 // this lane group's share, summed at the end
        // ---- P as two bf16 operands: P = hi + lo to about 2^-17 ----
        uint32_t ph[4], pl[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            ph[e2] = pack_bf16(pr[2 * e2], pr[2 * e2 + 1]);
            pl[e2] = pack_bf16(pr[2 * e2] - bf16_lo(ph[e2]), pr[2 * e2 + 1] - bf16_hi(ph[e2]));
        }
        const bf16x8 p_hi = __builtin_bit_cast(bf16x8, make_uint4(ph[0], ph[1], ph[2], ph[3]));
        const bf16x8 p_lo = __builtin_bit_cast(bf16x8, make_uint4(pl[0], pl[1], pl[2], pl[3]));
        // ---- V tile and the rescale factors cross lanes through LDS ----
        if (c4 == 0) sAlpha[w][n16] = alpha;
#pragma unroll
        for (int jj = 0; jj < NV; ++jj) *reinterpret_cast<u32x4*>(&sV[w][jj * 4 + c4][n16 * 8]) = vA[jj];
        if (LAZY) {       // ... and the V rows
#pragma unroll
            for (int jj = 0; jj < NV; ++jj) {
                const int row = r + jj * 4 + c4;
                if (row < n1) *reinterpret_cast<u32x4*>(const_cast<uint16_t*>(vb1) + (int64_t)row * kD + n16 * 8) = vA[jj];
            }
        }
        if (r_next < row1) load_v(r_next);
        wave_lds_sync();
        if (r != r_first && __any(alpha != 1.0f)) {     // the running max moved (first tile: the accumulators are still zero)
            const float4 al = *reinterpret_cast<const float4*>(&sAlpha[w][(c4 < NC ? c4 : 0) * 4]);
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                acc_o[dt][0] *= al.x; acc_o[dt][1] *= al.y; acc_o[dt][2] *= al.z; acc_o[dt][3] *= al.w;
            }
        }
        // ---- O += P V on the matrix cores, V operands by LDS transpose reads ----
        const uint16_t* vsrc = &sV[w][4 * c4 + (n16 >> 2)][4 * (n16 & 3)];
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            const v4s v0 = lds_read_tr16(vsrc + dt * 16);
            const v4s v1 = lds_read_tr16(vsrc + 16 * VS + dt * 16);
            const bf16x8 vb = __builtin_bit_cast(bf16x8, __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));
            acc_o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(p_hi, vb, acc_o[dt], 0, 0, 0);
            acc_o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(p_lo, vb, acc_o[dt], 0, 0, 0);
        }
        wave_lds_sync();      // sV / sAlpha are rewritten by the next tile
        return r_next;
    };

    {
        const int step = n_split * NW * ROWS;      // (== p.nch wherever a workgroup has a second tile, see active_workgroups)
        int r = r_first;
        if (r < row1) {
            // the early request stands unless part of this chunk maps to the tail of the full cache
            const bool spec_ok = spec && (!TWO_SEG || (c + 1) * NW * ROWS <= n1);
            if (!spec_ok) {
                load_k(r); load_v(r);
            } else if (r + ROWS > row1) {
                // early V rows past the end of the list hold whatever the cache holds there, maybe
                // NaN: P is 0 for them, but 0 * NaN is NaN, so they are cleared (early K rows need
                // nothing: their scores are replaced by -inf)
#pragma unroll
                for (int jj = 0; jj < NV; ++jj)
                    if (r + jj * 4 + c4 >= row1) vA[jj] = u32x4{0u, 0u, 0u, 0u};
            }
        }
        while (r < row1) r = compute_tile(r, r + step);
    }

    // ---- wavefront results to LDS ----
    l_run = sum_xor32(sum_xor16(l_run));
    if (c4 == 0) { sMw[w][n16] = m_run; sLw[w][n16] = l_run; }
    if (c4 < NC) {
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (4 * c4 + i < G) sO[w][4 * c4 + i][dt * 16 + n16] = acc_o[dt][i];
    }
    __syncthreads();

    // ---- merge the NW wavefronts and publish the partial result of this chunk ----
    const int64_t bg = (int64_t)b * p.Hkv + g;
    // what the NW wavefronts found for dims d, d + 1 of head gi, as one: max, sum, unnormalised output
    auto combine = [&](int gi, int d, float& M, float& L, float& acc0, float& acc1) {
        M = sMw[0][gi];
#pragma unroll
        for (int ww = 1; ww < NW; ++ww) M = fmaxf(M, sMw[ww][gi]);
        acc0 = 0.f; acc1 = 0.f; L = 0.f;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) {
            const float mw = sMw[ww][gi];
            const float sc = (mw == -INFINITY) ? 0.f : fast_exp2((mw - M) * kLog2e);
            const float2 t2 = *reinterpret_cast<const float2*>(&sO[ww][gi][d]);
            acc0 = fmaf(sc, t2.x, acc0);
            acc1 = fmaf(sc, t2.y, acc1);
            L = fmaf(sc, sLw[ww][gi], L);
        }
    };
    if (TAGGED) {
        // Wavefront w publishes the rows of heads w, w + NW: lane r < 43 dims 3r .. 3r + 2, lane 43 the
        // head's log-sum-exp.  The ticket is taken once every wavefront has ISSUED its rows; nothing
        // waits for their acknowledgement (hence a bare barrier: __syncthreads would wait for the stores).
        uint32_t* trows = p.tag_rows + (bg * kTagSlots + c_rec) * (G * kTagRowsPerHead * 4);
        const uint32_t tag = epoch + 1u != 0u ? epoch + 1u : 1u;           // this call's number: never 0
#pragma unroll
        for (int i = 0; i < UPW; ++i) {
            const int gi = w + i * NW;
            if (gi < G) {
                float M = sMw[0][gi];
#pragma unroll
                for (int ww = 1; ww < NW; ++ww) M = fmaxf(M, sMw[ww][gi]);
                const int d = 3 * min(lane, kTagDataRows - 1);
                float a0 = 0.f, a1 = 0.f, a2 = 0.f, L = 0.f;
#pragma unroll
                for (int ww = 0; ww < NW; ++ww) {
                    const float mw = sMw[ww][gi];
                    const float sc = (mw == -INFINITY) ? 0.f : fast_exp2((mw - M) * kLog2e);
                    a0 = fmaf(sc, sO[ww][gi][d], a0);
                    a1 = fmaf(sc, sO[ww][gi][d + 1], a1);
                    a2 = fmaf(sc, sO[ww][gi][min(d + 2, kD - 1)], a2);
                    L = fmaf(sc, sLw[ww][gi], L);
                }
                const float inv = L > 0.f ? __builtin_amdgcn_rcpf(L) : 0.f;
                const float lam = L > 0.f ? M + __logf(L) : -INFINITY;
                if (EMIT && lane == 0)
                    *reinterpret_cast<float2*>(p.part_ml + ((bg * kMaxChunks + c_rec) * G + gi) * 2) = make_float2(M, L);
                const bool lam_row = lane == kTagDataRows;
                if (lane <= kTagDataRows)
                    store_tagged_row(trows, G * kTagRowsPerHead, gi * kTagRowsPerHead + lane, lam_row ? lam : a0 * inv,
                                     lam_row ? 0.f : a1 * inv, (lam_row || d + 2 >= kD) ? 0.f : a2 * inv, tag);
            }
        }
        int32_t* counter = p.counters + bg * kCounterStride;
        // Merge by slices: every workgroup merges its share of the (head, data row) units, reading them from
        // all partial results as soon as its own are on their way; no workgroup waits for a ticket first, and
        // the merge is the work of all of them instead of one.  The ticket is still drawn: the workgroup that
        // publishes last does the bookkeeping, and takes over the slices of workgroups that gave up waiting
        // (words 2 and 3 of the counter line, as one: a bit per workgroup).  A workgroup gives up after slice_spin
        // re-reads, so that it never holds a compute unit that another workgroup of the launch is waiting for;
        // it then sets its bit and looks at the call number: still the old one, and the last workgroup has yet to
        // store it, which it does before it collects the bits, so it will see this one; already this call's, and
        // every workgroup has published, so the rows will arrive and the slice can be finished here after all
        // (if the last workgroup saw the bit as well, both write the same values).
        const bool slices = p.slice_merge != 0 && slices_fit;
        unsigned long long* pend = reinterpret_cast<unsigned long long*>(counter + 2);
        __shared__ unsigned long long sPend;
        asm volatile("s_barrier" ::: "memory");
        if (w == 0) {
            // the ticket, and for the workgroup that publishes last the bookkeeping, beside the merge of the slice
            int ticket = 0;
            if (lane == 0) ticket = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ticket = __builtin_amdgcn_readfirstlane(ticket);
            if (slices && ticket == nchunks - 1 && lane == 0) {
                __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);           // next call
                __hip_atomic_store(&p.epochs[bg], tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                wait_stores_acknowledged();                                                           // the call number is out before the bits are collected
                sPend = __hip_atomic_exchange(pend, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (lane == 0) sTicket = ticket;
        }
        if (slices && w == NW - 1) {
            const TagSlice sl = my_slice;
            if (sl.n_rows > 0 && !merge_tagged_slice_n<G>(p, b, g, tag_rsrc, sl, nchunks, tag, p.slice_spin, false)) {
                const unsigned long long bit = 1ull << c_rec;
                uint32_t seen = 0;
                if (lane == 0) {
                    const unsigned long long before = __hip_atomic_fetch_or(pend, bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    asm volatile("s_waitcnt vmcnt(0)" :: "v"(before) : "memory");       // the bit is set before the call number is read
                    seen = __hip_atomic_load(&p.epochs[bg], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                seen = __builtin_amdgcn_readfirstlane(seen);
                if (seen == tag) {
                    merge_tagged_slice_n<G>(p, b, g, tag_rsrc, sl, nchunks, tag, kTagSpinLimit, true);
                    if (lane == 0) __hip_atomic_fetch_and(pend, ~bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
        __syncthreads();
        if (sTicket != nchunks - 1) return;
        if (!slices) {
            // last arrival: every wavefront merges its heads
            merge_tagged_heads<G, UPW, (UPW == 1 ? 20 : 17)>(p, b, g, w, nchunks, tag);
            if (tid == 0) {
                __hip_atomic_store(&p.epochs[bg], tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);       // next call
            }
            return;
        }
        unsigned long long left = sPend;
        for (int k = 0; left != 0; ++k) {
            const int cb = __builtin_ctzll(left);
            left &= left - 1;
            TagSlice sl = tag_slice_of<G>(cb, nchunks);
            sl.gi = __builtin_amdgcn_readfirstlane(sl.gi); sl.r0 = __builtin_amdgcn_readfirstlane(sl.r0);
            sl.n_rows = __builtin_amdgcn_readfirstlane(sl.n_rows);
            if ((k & (NW - 1)) == w && cb < nchunks && sl.n_rows > 0)
                merge_tagged_slice_n<G>(p, b, g, tag_rsrc, sl, nchunks, tag, kTagSpinLimit, true);
        }
        return;
    }
    float* ml = p.part_ml + (bg * kMaxChunks + c_rec) * G * 2;
    float* po = p.part_o + (bg * p.max_chunks + c_rec) * G * kD;
    for (int e2 = tid; e2 < G * kD / 2; e2 += NT) {           // two consecutive dims per thread
        const int gi = (2 * e2) / kD, d = (2 * e2) % kD;
        float M, L, acc0, acc1;
        combine(gi, d, M, L, acc0, acc1);
        if (EMIT) {       // merged by the next kernel: ordinary stores
            *reinterpret_cast<float2*>(po + 2 * e2) = make_float2(acc0, acc1);
            if (d == 0) *reinterpret_cast<float2*>(ml + gi * 2) = make_float2(M, L);
        } else {
            coherent_store2(po + 2 * e2, acc0, acc1);
            if (d == 0) coherent_store2(ml + gi * 2, M, L);
        }
    }
    if (EMIT) return;

    // ---- ticketed hand-over: the workgroup that arrives last for (b, g) merges all chunks ----
    int32_t* counter = p.counters + bg * kCounterStride;
    wait_stores_acknowledged();
    __syncthreads();
    if (tid == 0) sTicket = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (sTicket != nchunks - 1) return;
    merge_partials<G, NW>(p, b, g, nchunks, &sO[0][0][0], &sO[0][0][0] + kMergeChunks * G, sMf, sLf);
    if (tid == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // next call
}

// Scores-only pass over the full cache (Section 4.3, "Impact of full attention steps", the
// "w/o full attention" setting: the attention scores over the entire cache are computed and the
// small cache is refreshed from them, but the step's output comes from the refreshed small cache,
// so V is never read here: half the bytes of a full step).  Same work split, K operand layout
// and score emission as attn_split_kernel; per workgroup it leaves only the (max, sum) pair of
// every head.  With no V registers to hold, two K tiles per wavefront are in flight.
template <int G>
__global__ __launch_bounds__(256, 3)
void score_split_kernel(const AttnParams p) {
    constexpr int NW = kSplitWaves, ROWS = kTileRows;
    const int c = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    if (p.pred != nullptr && p.pred[b] != p.pred_val) return;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n16 = lane & 15, c4 = lane >> 4;
    const int r_first = (c * NW + w) * ROWS;
    const int step = p.nch * NW * ROWS;
    const uint16_t* kb = p.k2 + (int64_t)b * p.s2_b + (int64_t)g * p.s2_h + c4 * 8;

    // first two tiles of this wavefront, requested before the length is known where they exist anyhow
    u32x4 kA[2][4], kB[2][4];
    const bool spec_a = (c + 1) * NW * ROWS <= p.cap2;
    const bool spec_b = (int64_t)r_first + step + ROWS <= p.cap2;
    auto load_exact = [&](u32x4 (&dst)[2][4], int r) {
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                dst[t][kk] = load_rows16<false>(kb + (int64_t)(r + t * 16 + n16) * kD + kk * 32);
    };
    if (spec_a) load_exact(kA, r_first);
    if (spec_b) load_exact(kB, r_first + step);

    bf16x8 qa[4];
    {
        const uint16_t* qrow = p.q + ((int64_t)b * p.Hq + (int64_t)g * G + (n16 < G ? n16 : 0)) * kD;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            uint4 u = *reinterpret_cast<const uint4*>(qrow + (kk * 4 + c4) * 8);
            if (n16 >= G) u = make_uint4(0, 0, 0, 0);
            qa[kk] = __builtin_bit_cast(bf16x8, u);
        }
    }
    const int n = min(max(min(p.seq_lens[b], p.cap2), 0), p.max_rows2);
    const int nchunks = active_workgroups(n, p.nch);
    if (c >= nchunks) return;
    auto load_clamped = [&](u32x4 (&dst)[2][4], int r) {     // rows past the end re-read the last row (masked later)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int row = min(r + t * 16 + n16, n - 1);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                dst[t][kk] = load_rows16<false>(kb + (int64_t)row * kD + kk * 32);
        }
    };
    float m_run = -INFINITY, l_run = 0.f;
    auto tile = [&](const u32x4 (&k)[2][4], int r) {
        float s[2][4];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k[t][kk]), qa[kk], acc, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 4; ++i) s[t][i] = (r + t * 16 + 4 * c4 + i < n) ? acc[i] * p.scale : -INFINITY;
        }
        if (n16 < G) {
            float* wrow = p.weights + ((int64_t)b * p.Hq + (int64_t)g * G + n16) * p.w_stride + r + 4 * c4;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int first = r + t * 16 + 4 * c4;
                if (p.w_vec && first + 4 <= n) {
                    *reinterpret_cast<float4*>(wrow + t * 16) = make_float4(s[t][0], s[t][1], s[t][2], s[t][3]);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (first + i < n) wrow[t * 16 + i] = s[t][i];
                }
            }
        }
        float mx = fmaxf(fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3])),
                         fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3])));
        mx = max_xor32(max_xor16(mx));
        const float m_new = fmaxf(m_run, mx);             // finite: the tile's first row is valid
        float ps = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ps += fast_exp2((s[e >> 2][e & 3] - m_new) * kLog2e);
        l_run = l_run * fast_exp2((m_run - m_new) * kLog2e) + ps;
        m_run = m_new;
    };
    // tiles alternate between the two register sets; each set is re-requested right after use
    int r = r_first;
    if (r < n && !spec_a) load_clamped(kA, r);
    if (r + step < n && !spec_b) load_clamped(kB, r + step);
    while (r < n) {
        tile(kA, r);
        if (r + 2 * step < n) load_clamped(kA, r + 2 * step);
        r += step;
        if (r >= n) break;
        tile(kB, r);
        if (r + 2 * step < n) load_clamped(kB, r + 2 * step);
        r += step;
    }
    l_run = sum_xor32(sum_xor16(l_run));
    __shared__ float sMw[NW][16], sLw[NW][16];
    if (c4 == 0) { sMw[w][n16] = m_run; sLw[w][n16] = l_run; }
    __syncthreads();
    if (tid < G) {
        float M = sMw[0][tid];
#pragma unroll
        for (int ww = 1; ww < NW; ++ww) M = fmaxf(M, sMw[ww][tid]);
        float L = 0.f;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) {
            const float mw = sMw[ww][tid];
            L = fmaf((mw == -INFINITY) ? 0.f : fast_exp2((mw - M) * kLog2e), sLw[ww][tid], L);
        }
        float* ml = p.part_ml + (((int64_t)b * p.Hkv + g) * kMaxChunks + c) * G * 2;
        *reinterpret_cast<float2*>(ml + tid * 2) = make_float2(M, L);
    }
}

// ---- pieces of the kernels that finish a full step whose scores were emitted ----
// LDS of one 256-thread workgroup that rebuilds lse of a query head and merges its output.
struct HeadMergeLds {
    __attribute__((aligned(8))) float red[8];
    float w[kMaxChunks];
    float lse[2];
    double L64;
    float acc[4][kD];
};
constexpr int kOutBatch = 24;                    // partial outputs per thread and round trip (96 partial results: one trip)

// lse of (b, h) in fp64 from the per-chunk (max, sum) pairs: s.lse = (hi, lo) with hi + lo = lse,
// s.w[c] = e^{m_c - M}, s.L64 = sum_c w_c l_c.  All 256 threads call; ends with a barrier.
// fp32_log: the caller only reports lse (to 1e-6) and normalises nothing by it: the logarithm, which one
// thread takes while all others wait, is the fp32 one (the fp64 library call costs 0.4 us there).
__device__ __forceinline__ void block_head_lse(const AttnParams& p, int G, int64_t bg, int gi, int nchunks,
                                               HeadMergeLds& s, bool fp32_log = false) {
    const int tid = threadIdx.x;
    const float* ml = p.part_ml + (bg * kMaxChunks * G + gi) * 2;
    float m = -INFINITY, l = 0.f;
    if (tid < nchunks) {                                   // nchunks <= kMaxChunks == blockDim
        const float2 t2 = *reinterpret_cast<const float2*>(ml + (int64_t)tid * G * 2);
        m = t2.x; l = t2.y;
    }
    const float M = block_max<4>(m, s.red);
    const float wgt = (m == -INFINITY) ? 0.f : fast_exp2((m - M) * kLog2e);
    if (tid < nchunks) s.w[tid] = wgt;
    const double L64 = block_sum_f64<4>((double)wgt * (double)l, reinterpret_cast<double*>(s.red));
    if (tid == 0) {
        float hi = -INFINITY, lo = 0.f;
        if (L64 > 0.0 && fp32_log) {
            hi = M + __logf((float)L64);
        } else if (L64 > 0.0) {
            const double l64 = (double)M + log(L64);
            hi = (float)l64;
            lo = (float)(l64 - (double)hi);
        }
        s.lse[0] = hi; s.lse[1] = lo; s.L64 = L64;
    }
    __syncthreads();
}

// First round of partial-output loads of (b, h); issued before block_head_lse so that the
// reductions there run under the memory latency.
__device__ __forceinline__ void head_out_request(const AttnParams& p, int G, int64_t bg, int gi, int nchunks,
                                                 float2 (&v)[kOutBatch]) {
    const int cg = threadIdx.x >> 6, d2 = threadIdx.x & 63;
    const float* po = p.part_o + (bg * p.max_chunks * G + gi) * kD + 2 * d2;
#pragma unroll
    for (int u = 0; u < kOutBatch; ++u)
        v[u] = *reinterpret_cast<const float2*>(po + (int64_t)min(cg + 4 * u, nchunks - 1) * G * kD);
}

// out[b,h,:] = sum_c w_c o_c[h,:] / L and lse[b,h]: four groups of 64 lanes take every fourth
// chunk.  Needs block_head_lse's results in s and head_out_request's in v.
__device__ __forceinline__ void block_head_out(const AttnParams& p, int G, int b, int64_t bg, int gi, int nchunks,
                                               HeadMergeLds& s, float2 (&v)[kOutBatch]) {
    const int tid = threadIdx.x, cg = tid >> 6, d2 = tid & 63;
    const int h = (int)(bg % p.Hkv) * G + gi;
    const float* po = p.part_o + (bg * p.max_chunks * G + gi) * kD + 2 * d2;
    float acc0 = 0.f, acc1 = 0.f;
    for (int c0 = cg; c0 < nchunks; c0 += 4 * kOutBatch) {
        if (c0 != cg) {
#pragma unroll
            for (int u = 0; u < kOutBatch; ++u)
                v[u] = *reinterpret_cast<const float2*>(po + (int64_t)min(c0 + 4 * u, nchunks - 1) * G * kD);
        }
#pragma unroll
        for (int u = 0; u < kOutBatch; ++u) {
            const float wc = (c0 + 4 * u < nchunks) ? s.w[c0 + 4 * u] : 0.f;
            acc0 = fmaf(wc, v[u].x, acc0);
            acc1 = fmaf(wc, v[u].y, acc1);
        }
    }
    s.acc[cg][2 * d2] = acc0; s.acc[cg][2 * d2 + 1] = acc1;
    __syncthreads();
    if (tid < kD) {
        const float L = (float)s.L64;
        const float o = L > 0.f ? (s.acc[0][tid] + s.acc[1][tid] + s.acc[2][tid] + s.acc[3][tid]) / L : 0.f;
        p.out[((int64_t)b * p.Hq + h) * kD + tid] = f32_to_bf16(o);
    }
    if (tid == 0) p.lse[(int64_t)b * p.Hq + h] = s.lse[0];
}

// weight = e^{s - lse} with lse = -nl + ll given as an fp32 pair.  The exponent is formed as an
// exact fp32 pair (two-sum) minus the low part of lse, so a weight carries the error of its
// score and of expf only (a plain fp32 subtraction alone would cost up to 5e-7 relative, which
// is the size of the gaps that decide the selection).
__device__ __forceinline__ float weight_of(float s, float nl, float ll) {
    const float hi = s + nl;
    const float bp = hi - s;
    const float lo = (s - (hi - bp)) + (nl - bp) - ll;     // s - lse = hi + lo, |lo| << 1
    const float e = expf(hi);
    return fmaf(e, lo, e);
}

// Second kernel of a full step that returns the attention weights.  Every workgroup first
// rebuilds lse of its (sequence, query head).  Workgroup x = 0 then merges the partial outputs of
// that head; workgroups x >= 1 turn kNormTile raw scores each into
// weights[b,h,j] = exp(s[b,h,j] - lse[b,h]), in place.
constexpr int kNormTile = 4096;

__global__ __launch_bounds__(256)
void merge_normalise_kernel(const AttnParams p, int G) {
    const int x = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    if (p.pred != nullptr && p.pred[b] != p.pred_val) return;
    const int tid = threadIdx.x;
    const int g = h / G, gi = h % G;
    const int len = min(max(min(p.seq_lens[b], p.cap2), 0), p.max_rows2);
    const int nchunks = p.ragged_batch != 0 ? ragged_chunks_of(p, b) : active_workgroups(len, p.nch);
    const int j0 = (x - 1) * kNormTile;
    if (x >= 1 && j0 >= len) return;

    __shared__ HeadMergeLds s;
    constexpr int PER = kNormTile / 256;         // scores per thread
    const int64_t bg = (int64_t)b * p.Hkv + g;
    float* row = p.weights + ((int64_t)b * p.Hq + h) * p.w_stride;

    // ---- request everything this workgroup needs before the first wait ----
    float sc[PER];
    float2 v[kOutBatch];
    if (x >= 1) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int j = j0 + i * 256 + tid;
            sc[i] = (j < len) ? row[j] : 0.f;
        }
    } else {
        head_out_request(p, G, bg, gi, nchunks, v);
    }
    block_head_lse(p, G, bg, gi, nchunks, s, p.weights == nullptr);       // (no weights: this is an output merge and nothing else)
    if (x == 0) {
        block_head_out(p, G, b, bg, gi, nchunks, s, v);
        return;
    }
    const float nl = -s.lse[0], ll = s.lse[1];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int j = j0 + i * 256 + tid;
        if (j < len) row[j] = weight_of(sc[i], nl, ll);
    }
}

// Second kernel of a full step that goes straight on to the selection (Section 2.2, "Decoding
// with full cache": the attention weights of the step decide the small cache).  Grid x < G: the
// output merge of query head x of the group, as above.  Grid x >= G: one tile of kPoolTile
// positions of one KV group: lse of all G heads (one wavefront per head), the weights of the
// tile and its pooling halo, their max over the group, the max-pool, and the first-level
// histogram of the selection.  Raw scores are read from `scores` (never modified, so the halo
// of a neighbouring tile is always raw); weights are written only if the caller wants them.
template <int G, int TILE>
__device__ __forceinline__
void finish_pool_body(const AttnParams& p, const float* __restrict__ scores, int64_t s_stride, int half, int agg,
                      float* __restrict__ pooled, int64_t pooled_stride, uint32_t* __restrict__ hist, const int b) {
    const int x = blockIdx.x, g = blockIdx.y;
    if (p.pred != nullptr && p.pred[b] != p.pred_val) return;
    const int tid = threadIdx.x;
    const int len = min(max(min(p.seq_lens[b], p.cap2), 0), p.max_rows2);
    const int nchunks = p.ragged_batch != 0 ? ragged_chunks_of(p, b) : active_workgroups(len, p.nch);
    const int64_t bg = (int64_t)b * p.Hkv + g;

    __shared__ HeadMergeLds s;
    const int n_merge = p.out != nullptr ? G : 0;     // no output to merge after a scores-only pass
    if (x < n_merge) {
        float2 v[kOutBatch];
        head_out_request(p, G, bg, x, nchunks, v);
        block_head_lse(p, G, bg, x, nchunks, s);
        block_head_out(p, G, b, bg, x, nchunks, s, v);
        return;
    }
    const int j0 = (x - n_merge) * TILE;
    if (j0 >= len && !(j0 == 0 && n_merge == 0)) return;   // (an empty sequence still gets its lse = -inf)

    __shared__ float sA[TILE + RK_MAX_POOL_W - 1];
    __shared__ uint32_t sH[kHistBins];
    __shared__ float sLse[G][2];
    constexpr int R = (TILE + RK_MAX_POOL_W - 1 + 255) / 256;
    const int span = TILE + 2 * half;
    const float* sg = scores + ((int64_t)b * p.Hq + (int64_t)g * G) * s_stride;

    // ---- request the raw scores of the tile and its halo, and the chunk statistics ----
    float sc[G][R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int i = r * 256 + tid, j = j0 - half + i;
        const bool in = i < span && j >= 0 && j < len;
        if (G == 4 && p.w_inter) {                  // the four heads of a position side by side: one 16-byte load
            const float4 v4 = in ? *reinterpret_cast<const float4*>(sg + (int64_t)j * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
            sc[0][r] = v4.x; sc[1 % G][r] = v4.y; sc[2 % G][r] = v4.z; sc[3 % G][r] = v4.w;
        } else {
#pragma unroll
            for (int gi = 0; gi < G; ++gi) sc[gi][r] = in ? sg[(int64_t)gi * s_stride + j] : 0.f;
        }
    }
    const int wv = tid >> 6, lane = tid & 63;
    constexpr int HPW = (G + 3) / 4;              // heads per wavefront
    constexpr int CPL = kMaxChunks / 64;          // chunk statistics per lane
    float m[HPW][CPL], l[HPW][CPL];
#pragma unroll
    for (int e = 0; e < HPW; ++e) {
        const int gi = wv + 4 * e;
        const float* ml = p.part_ml + (bg * kMaxChunks * G + min(gi, G - 1)) * 2;
#pragma unroll
        for (int u = 0; u < CPL; ++u) {
            const int c = lane + 64 * u;
            m[e][u] = -INFINITY; l[e][u] = 0.f;
            if (c < nchunks) {
                const float2 t2 = *reinterpret_cast<const float2*>(ml + (int64_t)c * G * 2);
                m[e][u] = t2.x; l[e][u] = t2.y;
            }
        }
    }
    for (int i = tid; i < kHistBins; i += 256) sH[i] = 0;

    // ---- lse of the G heads, fp64, one wavefront per head ----
#pragma unroll
    for (int e = 0; e < HPW; ++e) {
        const int gi = wv + 4 * e;
        float M = m[e][0];
#pragma unroll
        for (int u = 1; u < CPL; ++u) M = fmaxf(M, m[e][u]);
        M = wave_max(M);
        double L64 = 0.0;
#pragma unroll
        for (int u = 0; u < CPL; ++u) {
            const float wgt = (m[e][u] == -INFINITY) ? 0.f : fast_exp2((m[e][u] - M) * kLog2e);
            L64 += (double)wgt * (double)l[e][u];
        }
        L64 = wave_sum(L64);
        if (lane == 0 && gi < G) {
            float hi = -INFINITY, lo = 0.f;
            if (L64 > 0.0) {
                const double l64 = (double)M + log(L64);
                hi = (float)l64;
                lo = (float)(l64 - (double)hi);
            }
            sLse[gi][0] = hi; sLse[gi][1] = lo;
            if (n_merge == 0 && j0 == 0) p.lse[(int64_t)b * p.Hq + (int64_t)g * G + gi] = hi;
        }
    }
    __syncthreads();
    if (j0 >= len) return;

    // ---- weights, max over the group ----
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int i = r * 256 + tid, j = j0 - half + i;
        if (i < span) {
            float a = -INFINITY;                     // outside [0, len): never wins a max
            if (j >= 0 && j < len) {
                const bool core = p.weights != nullptr && i >= half && i < half + TILE;
#pragma unroll
                for (int gi = 0; gi < G; ++gi) {
                    const float wgt = weight_of(sc[gi][r], -sLse[gi][0], sLse[gi][1]);
                    if (core) p.weights[((int64_t)b * p.Hq + (int64_t)g * G + gi) * p.w_stride + j] = wgt;
                    a = aggregate(a, wgt, gi, agg);
                }
                if (agg == RK_AGG_MEAN) a = __fdiv_rn(a, (float)G);
            }
            sA[i] = a;
        }
    }
    __syncthreads();

    // ---- max-pool, store, histogram ----
    float* prow = pooled + bg * pooled_stride;
    for (int i = tid; i < TILE; i += 256) {
        const int j = j0 + i;
        if (j < len) {
            float mx = sA[i];
            for (int d = 1; d <= 2 * half; ++d) mx = fmaxf(mx, sA[i + d]);
            mx += 0.0f;                           // -0 becomes +0: one bit pattern per value
            prow[j] = mx;
            atomicAdd(&sH[key_of(mx) >> kHistShift], 1u);
        }
    }
    __syncthreads();
    uint32_t* gh = hist + bg * kHistBins;
    for (int i = tid; i < kHistBins; i += 256) {
        const uint32_t c = sH[i];
        if (c != 0) atomicAdd(&gh[i], c);
    }
}

template <int G, int TILE>
__global__ __launch_bounds__(256, G <= 4 ? 5 : 1)       // (as pool_batched_kernel below: full step with selection at 131072 rows 144 -> 141 us)
void finish_pool_kernel(const AttnParams p, const float* __restrict__ scores, int64_t s_stride, int half, int agg,
                        float* __restrict__ pooled, int64_t pooled_stride, uint32_t* __restrict__ hist) {
    finish_pool_body<G, TILE>(p, scores, s_stride, half, agg, pooled, pooled_stride, hist, (int)blockIdx.z);
}

// The pooling half of the finishing kernel for several layers in one launch (grid z = layer *
// batch + sequence): each layer's raw scores and chunk statistics are where its full attention
// left them, in a workspace of its own.  What differs from layer to layer comes from a table
// passed by value.
// With many layers in one launch the workgroups come in rounds and each pays its own chain of
// round trips (statistics, lse, scores, histogram): larger tiles, fewer rounds.
constexpr int kBatchedPoolTile = 2048;       // (the launch alone, 32 layers of 33k rows or 8 of 131k: 1024: 81, 2048: 72, 4096: 85, 8192: 103 us)

struct PoolBatch {
    const float* part_ml[kBatchLayers];
    const float* scores[kBatchLayers];
    float* lse[kBatchLayers];
    float* pooled[kBatchLayers];
    uint32_t* hist[kBatchLayers];
    const int32_t* pred[kBatchLayers];       // NULL: every sequence of the layer
};

// (Groups of up to 4 heads are compiled for 5 workgroups per CU: a workgroup is a chain of phases, each
// waiting on the one before, and more of them in flight fill the waits: 72 -> 66 us per launch over 32
// layers of 33k rows; for 6 it spills and gains nothing more, for 8: 75 us.  Larger groups hold more scores per thread.)
template <int G>
__global__ __launch_bounds__(256, G <= 4 ? 5 : 1)
void pool_batched_kernel(const PoolBatch tab, const AttnParams common, int32_t batch, int64_t stride, int half, int agg) {
    const int layer = blockIdx.z / batch, b = blockIdx.z - layer * batch;
    AttnParams p = common;                   // out == NULL and weights == NULL: pooling tiles only
    p.part_ml = const_cast<float*>(tab.part_ml[layer]);
    p.lse = tab.lse[layer];
    p.pred = tab.pred[layer];
    finish_pool_body<G, kBatchedPoolTile>(p, tab.scores[layer], stride, half, agg, tab.pooled[layer], stride, tab.hist[layer], b);
}

template <int G>
static int launch_pool_batched(const PoolBatch& tab, const AttnParams& p, int n, int batch, int32_t max_len, int half,
                               int agg, hipStream_t st) {
    dim3 grid((max_len + kBatchedPoolTile - 1) / kBatchedPoolTile, p.Hkv, n * batch);
    hipLaunchKernelGGL((pool_batched_kernel<G>), grid, dim3(256), 0, st, tab, p, (int32_t)batch,
                       pooled_row_stride(max_len), half, agg);
    return launch_status();
}

template <int G>
static int launch_finish_pool(const AttnParams& p, int batch, int32_t max_len, const Workspace& ws, int half, int agg,
                              hipStream_t st) {
    const int tile = pool_tile_for(max_len);
    dim3 grid((p.out != nullptr ? G : 0) + (max_len + tile - 1) / tile, p.Hkv, batch);
    const int64_t stride = pooled_row_stride(max_len);
    if (tile == kPoolTileLong)
        hipLaunchKernelGGL((finish_pool_kernel<G, kPoolTileLong>), grid, dim3(256), 0, st, p, ws.scores, stride, half, agg, ws.pooled, stride, ws.hist);
    else
        hipLaunchKernelGGL((finish_pool_kernel<G, kPoolTile>), grid, dim3(256), 0, st, p, ws.scores, stride, half, agg, ws.pooled, stride, ws.hist);
    return launch_status();
}

// Merge by slices (see the kernel) where every workgroup of the launch is resident at once: the kernels are
// compiled for at least two workgroups per compute unit.  A larger launch keeps the merge by the last workgroup,
// which waits for nobody.  g_slice_spin: how often a workgroup re-reads rows that are still in flight before it
// leaves its slice to the last one (rk_debug_set_slice_spin: a test hook; 0 makes every workgroup give up at once).
static std::atomic<int32_t> g_slice_spin{256};
static void set_slice_merge(AttnParams& p, bool tagged, int64_t workgroups) {
    p.slice_merge = (tagged && workgroups <= 2 * kComputeUnits) ? 1 : 0;
    p.slice_spin = g_slice_spin.load(std::memory_order_relaxed);
}

template <int G, bool EMIT, bool TWO_SEG, bool TAGGED, bool TRIG = false>
static int launch_split_g(const AttnParams& p, int batch, int nchunk_grid, hipStream_t st) {
    // (measured on the kernel alone, us per launch, chunk as grid x / KV head as grid x: 8 KV heads, 512
    // workgroups, 32768..33000 rows 25.8 - 29.2 / 25.2 - 26.0; 4 KV heads, 65536..65800 rows 27.0 - 32.7 /
    // 27.0 - 29.7; 8 KV heads, 1024 workgroups, which are not all resident at once, 131072..131400 rows
    // 101.3 - 105.4 / 105.5; no difference at 8192 and 16384 rows)
    const bool heads_first = EMIT && !TWO_SEG && p.ragged_batch == 0 &&
                             (int64_t)nchunk_grid * p.Hkv * batch <= 3 * kComputeUnits;
    dim3 grid(heads_first ? p.Hkv : nchunk_grid, heads_first ? batch : p.Hkv, heads_first ? nchunk_grid : batch);
    // four wavefronts of 32 rows per iteration; with 64-row chunks two of them only help to merge
    const int32_t spec_rows = TWO_SEG ? (p.n_sel < p.cap1 ? p.n_sel : p.cap1) : p.cap2;
    const int64_t tail_c = (TWO_SEG && p.tail_wg) ? p.nch : heads_first ? kHeadsFirst : kNoTailWg;
    // (TRIG: the pointers the test needs first travel in the preloaded slots of the predicate and the call numbers)
    hipLaunchKernelGGL((attn_split_kernel<G, 4, EMIT, TWO_SEG, false, TAGGED, TRIG>), grid, dim3(256), 0, st,
                       TWO_SEG ? p.k1 : p.k2, TWO_SEG ? p.v1 : p.v2, (TWO_SEG ? p.s1_b : p.s2_b) | (tail_c << 56),
                       (int32_t)(TWO_SEG ? p.s1_h : p.s2_h), spec_rows, p.seq_lens, p.tail_start,
                       TRIG ? reinterpret_cast<const int32_t*>(p.q) : p.pred,
                       TRIG ? reinterpret_cast<const uint32_t*>(p.trig_q_ref) : p.epochs, p);
    return launch_status();
}

template <int G>
static int launch_lazy_g(const AttnParams& p, int batch, hipStream_t st) {
    dim3 grid(p.nch, p.Hkv, batch);
    hipLaunchKernelGGL((attn_split_kernel<G, 4, false, true, true>), grid, dim3(256), 0, st,
                       p.k2, p.v2, p.s2_b | ((int64_t)kNoTailWg << 56), (int32_t)p.s2_h, p.n_sel, p.seq_lens, p.tail_start, p.idx, p.epochs, p);
    return launch_status();
}

static int launch_lazy(const AttnParams& p, int batch, int G, hipStream_t st) {
    switch (G) {
        case 1: return launch_lazy_g<1>(p, batch, st);
        case 2: return launch_lazy_g<2>(p, batch, st);
        case 3: return launch_lazy_g<3>(p, batch, st);
        case 4: return launch_lazy_g<4>(p, batch, st);
        case 5: return launch_lazy_g<5>(p, batch, st);
        case 6: return launch_lazy_g<6>(p, batch, st);
        case 7: return launch_lazy_g<7>(p, batch, st);
        case 8: return launch_lazy_g<8>(p, batch, st);
        default: return RK_ERR_UNSUPPORTED;
    }
}

template <bool EMIT, bool TWO_SEG, bool TAGGED = !EMIT>
static int launch_split(const AttnParams& p, int batch, int G, int nchunk_grid, hipStream_t st) {
    switch (G) {
        case 1: return launch_split_g<1, EMIT, TWO_SEG, TAGGED>(p, batch, nchunk_grid, st);
        case 2: return launch_split_g<2, EMIT, TWO_SEG, TAGGED>(p, batch, nchunk_grid, st);
        case 3: return launch_split_g<3, EMIT, TWO_SEG, TAGGED>(p, batch, nchunk_grid, st);
        case 4: return launch_split_g<4, EMIT, TWO_SEG, TAGGED>(p, batch, nchunk_grid, st);
        case 5: return launch_split_g<5, EMIT, TWO_SEG, TAGGED>(p, batch, nchunk_grid, st);
        case 6: return launch_split_g<6, EMIT, TWO_SEG, TAGGED>(p, batch, nchunk_grid, st);
        case 7: return launch_split_g<7, EMIT, TWO_SEG, TAGGED>(p, batch, nchunk_grid, st);
        case 8: return launch_split_g<8, EMIT, TWO_SEG, TAGGED>(p, batch, nchunk_grid, st);
        default: return RK_ERR_UNSUPPORTED;
    }
}

// The partial step that tests the trigger itself: tagged hand-over for groups of up to 4 heads; beyond, tagged
// where the merge by slices applies and ticketed otherwise (as without the trigger, see launch_partial).
static int launch_split_triggered(const AttnParams& p, int batch, int G, int nchunk_grid, bool tagged, hipStream_t st) {
    switch (G) {
        case 1: return launch_split_g<1, false, true, true, true>(p, batch, nchunk_grid, st);
        case 2: return launch_split_g<2, false, true, true, true>(p, batch, nchunk_grid, st);
        case 3: return launch_split_g<3, false, true, true, true>(p, batch, nchunk_grid, st);
        case 4: return launch_split_g<4, false, true, true, true>(p, batch, nchunk_grid, st);
#define RK_CASE(g) case g: return tagged ? launch_split_g<g, false, true, true, true>(p, batch, nchunk_grid, st) \
                                         : launch_split_g<g, false, true, false, true>(p, batch, nchunk_grid, st);
        RK_CASE(5) RK_CASE(6) RK_CASE(7) RK_CASE(8)
#undef RK_CASE
        default: return RK_ERR_UNSUPPORTED;
    }
}

static int launch_score_split(const AttnParams& p, int batch, int G, int nchunk_grid, hipStream_t st) {
    dim3 grid(nchunk_grid, p.Hkv, batch);
    switch (G) {
#define RK_CASE(g) case g: hipLaunchKernelGGL((score_split_kernel<g>), grid, dim3(256), 0, st, p); break;
        RK_CASE(1) RK_CASE(2) RK_CASE(3) RK_CASE(4) RK_CASE(5) RK_CASE(6) RK_CASE(7) RK_CASE(8)
#undef RK_CASE
        default: return RK_ERR_UNSUPPORTED;
    }
    return launch_status();
}

int full_attn_stage(const rk_geom* geom, const void* q, rk_kv full, const int32_t* seq_lens, int32_t max_len,
                    void* out, float* weights, int64_t w_stride, float* lse, const int32_t* pred, int32_t pred_val,
                    const Workspace& ws, hipStream_t st, bool scores_only, int pool_half, bool no_v, int agg,
                    bool co_run, bool defer_pool) {
    const int G = geom->n_q_heads / geom->n_kv_heads;
    const bool fused = pool_half >= 0;
    const bool emit = weights != nullptr || fused;
    AttnParams p{};
    p.q = (const uint16_t*)q;
    p.k2 = (const uint16_t*)full.k; p.v2 = (const uint16_t*)full.v;
    p.s2_b = full.stride_b; p.s2_h = full.stride_h;
    p.seq_lens = seq_lens;
    p.n_sel = 0;
    p.max_rows2 = max_len;
    p.cap1 = 0; p.cap2 = (int32_t)full.capacity;
    p.nch = emit ? emit_split_workgroups(geom, max_len)
                 : split_workgroups(max_len, (int64_t)geom->batch * geom->n_kv_heads, kMergeChunks);
    if (co_run) {       // more, smaller workgroups, unless that means more partial results than the finish takes cheaply
        const int wide = split_workgroups(max_len, (int64_t)geom->batch * geom->n_kv_heads, kMaxChunks, kCoRunTargetWgs);
        if (wide <= kCoRunMaxChunks) p.nch = wide;
    }
    p.Hq = geom->n_q_heads; p.Hkv = geom->n_kv_heads;
    p.scale = geom->scale;
    p.out = (uint16_t*)out;
    if (fused) { p.weights = ws.scores; p.w_stride = pooled_row_stride(max_len); p.w_inter = (G == 4 && !no_v) ? 1 : 0; }
    else       { p.weights = weights;   p.w_stride = w_stride; }
    p.w_vec = (p.weights && (p.w_stride % 4 == 0) && aligned16(p.weights)) ? 1 : 0;
    p.lse = lse ? lse : ws.lse;
    p.pred = pred; p.pred_val = pred_val;
    p.counters = ws.counters; p.part_ml = ws.part_ml; p.part_o = ws.part_o; p.max_chunks = ws.max_chunks;
    p.epochs = ws.epochs; p.tag_rows = ws.tag_rows;
    p.ragged_batch = (emit && !no_v) ? ragged_batch_of(geom) : 0;
    if (!emit) {
        // No scores wanted.  Short rows: one launch, merged by the last workgroup inside it (at most
        // kMergeChunks partial results).  Long rows: the wider split of the score-emitting kernel
        // (its stores switched off) and the merge as a second small launch fill the chip better.
        const int wide = split_workgroups(max_len, (int64_t)geom->batch * geom->n_kv_heads, kMaxChunks);
        if (wide <= kMergeChunks) {
            const int64_t problems = (int64_t)geom->batch * geom->n_kv_heads;
            int own = 0;
            p.nch = (ws.tag_rows != nullptr && problems <= 8) ? sliced_split_workgroups(max_len, 0, &own, problems, kSliceChunks4)
                                                              : merged_split_workgroups(max_len, 0, problems);
            set_slice_merge(p, true, (int64_t)p.nch * problems);
            return launch_split<false, false>(p, geom->batch, G, p.nch, st);
        }
        p.nch = wide;
        p.weights = nullptr;
        p.ragged_batch = ragged_batch_of(geom);
        int rc = launch_split<true, false>(p, geom->batch, G, p.nch, st);
        if (rc != RK_OK) return rc;
        hipLaunchKernelGGL(merge_normalise_kernel, dim3(1, geom->n_q_heads, geom->batch), dim3(256), 0, st, p, G);
        return launch_status();
    }
    const int nchunk_grid = p.nch;
    // Where the pooling is deferred, nothing but the output merge would follow this kernel at once: it is merged
    // inside the kernel instead of by a launch that waits for this one (tagged partial results, merged by slices, as
    // in the partial step; full step of 32 heads over 32768 rows: 36.8 -> 35.7 us per layer).  Groups of up to 4 heads,
    // all workgroups of the launch resident at once, no more partial results than that merge takes.  (Where the
    // finish follows at once its first workgroups merge the output beside the pooling tiles, which costs nothing;
    // merged inside, that step was 2.5 us slower.)
    const bool merge_inside = fused && defer_pool && !no_v && !scores_only && ws.tag_rows != nullptr && G <= kSplitWaves && p.ragged_batch == 0 &&
                              nchunk_grid <= kSliceChunks4 &&
                              (int64_t)nchunk_grid * geom->batch * geom->n_kv_heads <= 2 * kComputeUnits;
    int rc;
    if (merge_inside) {
        set_slice_merge(p, true, (int64_t)nchunk_grid * geom->batch * geom->n_kv_heads);
        switch (G) {
            case 1: rc = launch_split_g<1, true, false, true>(p, geom->batch, nchunk_grid, st); break;
            case 2: rc = launch_split_g<2, true, false, true>(p, geom->batch, nchunk_grid, st); break;
            case 3: rc = launch_split_g<3, true, false, true>(p, geom->batch, nchunk_grid, st); break;
            default: rc = launch_split_g<4, true, false, true>(p, geom->batch, nchunk_grid, st); break;
        }
    } else {
        rc = no_v ? launch_score_split(p, geom->batch, G, nchunk_grid, st)
                  : launch_split<true, false>(p, geom->batch, G, nchunk_grid, st);
    }
    if (rc != RK_OK || scores_only) return rc;
    if (!fused) {
        dim3 grid(1 + (max_len + kNormTile - 1) / kNormTile, geom->n_q_heads, geom->batch);
        hipLaunchKernelGGL(merge_normalise_kernel, grid, dim3(256), 0, st, p, G);
        return launch_status();
    }
    if (defer_pool) {            // only the output is finished now; pool_batched_stage does the rest later
        if (merge_inside) return rc;
        p.weights = nullptr;
        hipLaunchKernelGGL(merge_normalise_kernel, dim3(1, geom->n_q_heads, geom->batch), dim3(256), 0, st, p, G);
        return launch_status();
    }
    p.weights = weights; p.w_stride = w_stride;          // where the finish writes weights, if anywhere
    switch (G) {
        case 1: return launch_finish_pool<1>(p, geom->batch, max_len, ws, pool_half, agg, st);
        case 2: return launch_finish_pool<2>(p, geom->batch, max_len, ws, pool_half, agg, st);
        case 3: return launch_finish_pool<3>(p, geom->batch, max_len, ws, pool_half, agg, st);
        case 4: return launch_finish_pool<4>(p, geom->batch, max_len, ws, pool_half, agg, st);
        case 5: return launch_finish_pool<5>(p, geom->batch, max_len, ws, pool_half, agg, st);
        case 6: return launch_finish_pool<6>(p, geom->batch, max_len, ws, pool_half, agg, st);
        case 7: return launch_finish_pool<7>(p, geom->batch, max_len, ws, pool_half, agg, st);
        case 8: return launch_finish_pool<8>(p, geom->batch, max_len, ws, pool_half, agg, st);
        default: return RK_ERR_UNSUPPORTED;
    }
}

// The pooled scores and histograms of n_layers layers whose full attention ran with defer_pool,
// each on its own workspace, with the launch shape emit_split_workgroups gives.
int pool_batched_stage(const rk_geom* geom, int n_layers, const Workspace* wss, const int32_t* seq_lens, int32_t max_len,
                       int64_t full_capacity, int pool_half, int agg, const int32_t* const* pred, int32_t pred_val,
                       hipStream_t st) {
    const int G = geom->n_q_heads / geom->n_kv_heads;
    if ((int64_t)kBatchLayers * geom->batch > 65535) return RK_ERR_UNSUPPORTED;
    AttnParams p{};
    p.seq_lens = seq_lens;
    p.max_rows2 = max_len;
    p.cap2 = (int32_t)full_capacity;
    p.nch = emit_split_workgroups(geom, max_len);
    p.ragged_batch = ragged_batch_of(geom);
    p.Hq = geom->n_q_heads; p.Hkv = geom->n_kv_heads;
    p.w_inter = G == 4 ? 1 : 0;              // how full_attn_stage(defer_pool) left the raw scores
    p.pred_val = pred_val;
    for (int l0 = 0; l0 < n_layers; l0 += kBatchLayers) {
        const int n = n_layers - l0 < kBatchLayers ? n_layers - l0 : kBatchLayers;
        PoolBatch tab{};
        for (int l = 0; l < n; ++l) {
            const Workspace& w = wss[l0 + l];
            tab.part_ml[l] = w.part_ml; tab.scores[l] = w.scores; tab.lse[l] = w.lse;
            tab.pooled[l] = w.pooled; tab.hist[l] = w.hist;
            tab.pred[l] = pred ? pred[l0 + l] : nullptr;
        }
        int rc;
        switch (G) {
            case 1: rc = launch_pool_batched<1>(tab, p, n, geom->batch, max_len, pool_half, agg, st); break;
            case 2: rc = launch_pool_batched<2>(tab, p, n, geom->batch, max_len, pool_half, agg, st); break;
            case 3: rc = launch_pool_batched<3>(tab, p, n, geom->batch, max_len, pool_half, agg, st); break;
            case 4: rc = launch_pool_batched<4>(tab, p, n, geom->batch, max_len, pool_half, agg, st); break;
            case 5: rc = launch_pool_batched<5>(tab, p, n, geom->batch, max_len, pool_half, agg, st); break;
            case 6: rc = launch_pool_batched<6>(tab, p, n, geom->batch, max_len, pool_half, agg, st); break;
            case 7: rc = launch_pool_batched<7>(tab, p, n, geom->batch, max_len, pool_half, agg, st); break;
            case 8: rc = launch_pool_batched<8>(tab, p, n, geom->batch, max_len, pool_half, agg, st); break;
            default: return RK_ERR_UNSUPPORTED;
        }
        if (rc != RK_OK) return rc;
    }
    return RK_OK;
}

}  // namespace rk

using namespace rk;

static int check_full_args(const rk_geom* geom, const void* q, rk_kv full, const int32_t* seq_lens, int32_t max_len,
                           void* out, bool need_out, float* weights, int64_t w_stride) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!q || (!out && need_out) || !seq_lens || max_len <= 0) return RK_ERR_INVALID_ARG;
    if (!aligned16(q) || ((uintptr_t)out & 1u)) return RK_ERR_INVALID_ARG;
    if ((rc = check_kv(full)) != RK_OK) return rc;
    if (weights && (w_stride < max_len || ((uintptr_t)weights & 3u))) return RK_ERR_INVALID_ARG;
    return RK_OK;
}

extern "C" int rk_full_attn(const rk_geom* geom, const void* q, rk_kv full,
                            const int32_t* seq_lens, int32_t max_len,
                            void* out, float* weights, int64_t w_stride, float* lse,
                            const int32_t* pred, int32_t pred_val,
                            void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_full_args(geom, q, full, seq_lens, max_len, out, true, weights, w_stride);
    if (rc != RK_OK) return rc;
    Workspace ws;
    if ((rc = check_workspace(geom, max_len, 0, workspace, workspace_bytes, &ws)) != RK_OK) return rc;
    return full_attn_stage(geom, q, full, seq_lens, max_len, out, weights, w_stride, lse, pred, pred_val,
                           ws, (hipStream_t)stream, false, -1, false, RK_AGG_MAX);
}

extern "C" int rk_full_attn_scores(const rk_geom* geom, const void* q, rk_kv full,
                                   const int32_t* seq_lens, int32_t max_len,
                                   float* scores, int64_t s_stride,
                                   const int32_t* pred, int32_t pred_val,
                                   void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_full_args(geom, q, full, seq_lens, max_len, nullptr, false, scores, s_stride);
    if (rc != RK_OK) return rc;
    Workspace ws;
    if ((rc = check_workspace(geom, max_len, 0, workspace, workspace_bytes, &ws)) != RK_OK) return rc;
    // scores == NULL: the kernel exactly as a full step of rk_full_attn_select / rk_full_attn_deferred
    // launches it, the raw scores going to the workspace in the library's own arrangement
    return full_attn_stage(geom, q, full, seq_lens, max_len, nullptr, scores, s_stride, nullptr, pred, pred_val,
                           ws, (hipStream_t)stream, true, scores ? -1 : 0, false, RK_AGG_MAX);
}

// Argument checks of the partial step (everything but the scratch memory).
static int check_partial_args(const rk_geom* geom, const void* q, rk_kv small, int32_t n_sel, rk_kv full,
                              const int32_t* tail_start, const int32_t* seq_lens, int32_t max_recent, void* out) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!q || !out || !seq_lens || !tail_start || n_sel < 0 || max_recent < 0) return RK_ERR_INVALID_ARG;
    if (n_sel + (int64_t)max_recent <= 0 || n_sel + (int64_t)max_recent > INT32_MAX) return RK_ERR_INVALID_ARG;
    if (!aligned16(q) || ((uintptr_t)out & 1u)) return RK_ERR_INVALID_ARG;
    if ((rc = check_kv(full)) != RK_OK) return rc;
    if (n_sel > 0 && (rc = check_kv(small)) != RK_OK) return rc;
    return RK_OK;
}

// The query-similarity test a partial step carries out itself (rk_partial_attn_triggered).
struct Trigger { float* q_ref; float threshold; float* sim; int32_t* need_full; };

// Launch of the partial step; `ws` needs counters, lse, part_ml, part_o and max_chunks only.
static int launch_partial(const rk_geom* geom, const void* q, rk_kv small, int32_t n_sel, bool evict,
                          rk_kv full, const int32_t* tail_start, const int32_t* seq_lens,
                          int32_t max_recent, void* out, const int32_t* pred, int32_t pred_val,
                          const Workspace& ws, void* stream, const int32_t* lazy_idx = nullptr,
                          const Trigger* trig = nullptr) {
    const int G = geom->n_q_heads / geom->n_kv_heads;
    AttnParams p{};
    p.q = (const uint16_t*)q;
    p.k1 = (const uint16_t*)small.k; p.v1 = (const uint16_t*)small.v;
    p.s1_b = small.stride_b; p.s1_h = small.stride_h;
    p.k2 = (const uint16_t*)full.k; p.v2 = (const uint16_t*)full.v;
    p.s2_b = full.stride_b; p.s2_h = full.stride_h;
    p.tail_start = tail_start;
    p.seq_lens = seq_lens;
    p.n_sel = n_sel;
    p.evict = evict ? 1 : 0;
    p.max_rows2 = max_recent;
    p.cap1 = n_sel > 0 ? (int32_t)small.capacity : 0; p.cap2 = (int32_t)full.capacity;
    p.Hq = geom->n_q_heads; p.Hkv = geom->n_kv_heads;
    p.scale = geom->scale;
    p.out = (uint16_t*)out;
    p.lse = ws.lse;
    p.pred = pred; p.pred_val = pred_val;
    p.counters = ws.counters; p.part_ml = ws.part_ml; p.part_o = ws.part_o; p.max_chunks = ws.max_chunks;
    p.epochs = ws.epochs; p.tag_rows = ws.tag_rows;
    // Which hand-over.  Tagged partial results merged by slices (every workgroup its share, see the kernel) wherever
    // that merge applies: a launch whose workgroups are all resident at once, with no more partial results per
    // (sequence, KV head) than it has a form for.  Otherwise: rows enough for 32 workgroups per pair of a launch over
    // few pairs take the ticketed form with two batches of partial results (see two_batches_pay); groups of up to 4
    // heads the tagged form merged by the last workgroup, one head per wavefront; larger groups the ticketed form
    // (two heads per wavefront: measured at 7 heads per group, 4096 rows, 9.9 against 10.7 us).
    const int64_t problems = (int64_t)geom->batch * geom->n_kv_heads;
    const bool can_tag = ws.tag_rows != nullptr;                                       // (the built-in scratch array has no tagged region)
    // a few rows decoded since the refresh: a workgroup of their own (see the kernel), the others split the small cache
    // (ticketed merge: a 17th partial result costs it a second round trip, more than the tail workgroup gains)
    int tail_wg_tagged = (can_tag && lazy_idx == nullptr && n_sel > 0 && max_recent <= kMinChunk) ? 1 : 0;
    int nch_tagged;
    if (lazy_idx == nullptr && problems >= 16) {                                       // many (sequence, KV head) pairs: see there
        if (tail_wg_tagged) nch_tagged = batched_tagged_workgroups(n_sel, max_recent, &tail_wg_tagged, problems);
        else nch_tagged = batched_tagged_workgroups(n_sel + (int64_t)max_recent, 0, &tail_wg_tagged, problems);
    } else if (lazy_idx == nullptr && can_tag && problems <= 8) {                      // few pairs: sized for the merge by slices
        nch_tagged = sliced_split_workgroups(n_sel, max_recent, &tail_wg_tagged, problems, kSliceChunks4);
    } else {
        nch_tagged = merged_split_workgroups(n_sel, tail_wg_tagged ? 0 : max_recent, problems, false);
    }
    // (larger groups, whose wavefronts publish two heads each: only where the launch is a matter of latency, few
    // pairs; measured at 7 and 8 heads per group, 2048 rows: 32 pairs 13.5 -> 14.9 us, 64 pairs 19.5 -> 21.4,
    // against 16 pairs of 4096 rows 13.1 -> 12.6 and 4 pairs 9.7 -> 9.0)
    const bool by_slices = can_tag && nch_tagged + tail_wg_tagged <= kSliceChunks4 &&
                           (int64_t)(nch_tagged + tail_wg_tagged) * problems <= 2 * kComputeUnits &&
                           (G <= kSplitWaves || problems <= 16);
    const bool wide = !by_slices && lazy_idx == nullptr && trig == nullptr && two_batches_pay(n_sel, max_recent, problems);
    const bool tagged = can_tag && !wide && (by_slices || G <= kSplitWaves);
    p.tail_wg = tagged ? tail_wg_tagged : 0;
    p.nch = tagged ? nch_tagged
                   : merged_split_workgroups(n_sel, max_recent, problems, lazy_idx == nullptr && (trig == nullptr || G > kSplitWaves));
    if (!tagged && p.nch > p.max_chunks) p.nch = p.max_chunks;      // fewer, longer chunks: what the workspace has slots for
    if (p.nch > kMergeChunks || p.nch < 1) return RK_ERR_WORKSPACE;
    set_slice_merge(p, tagged, (int64_t)(p.nch + (lazy_idx == nullptr ? p.tail_wg : 0)) * problems);
    if (lazy_idx != nullptr) {      // rows of the selection come from the full cache and are written to `small` on the way
        if (n_sel < 1 || small.capacity < n_sel) return RK_ERR_INVALID_ARG;
        p.idx = lazy_idx; p.idx_stride = n_sel;
        return launch_lazy(p, geom->batch, G, (hipStream_t)stream);
    }
    const int nchunk_grid = p.nch + p.tail_wg;
    if (trig != nullptr) {
        if (ws.tag_rows == nullptr || pred != nullptr) return RK_ERR_INVALID_ARG;
        p.trig_q_ref = trig->q_ref; p.trig_sim = trig->sim; p.trig_need = trig->need_full; p.trig_threshold = trig->threshold;
        return launch_split_triggered(p, geom->batch, G, nchunk_grid, tagged, (hipStream_t)stream);
    }
    if (!tagged) return launch_split<false, true, false>(p, geom->batch, G, nchunk_grid, (hipStream_t)stream);
    return launch_split<false, true>(p, geom->batch, G, nchunk_grid, (hipStream_t)stream);
}

static int partial_attn_impl(const rk_geom* geom, const void* q, rk_kv small, int32_t n_sel, bool evict,
                             rk_kv full, const int32_t* tail_start, const int32_t* seq_lens,
                             int32_t max_recent, void* out,
                             const int32_t* pred, int32_t pred_val,
                             void* workspace, size_t workspace_bytes, void* stream, const int32_t* lazy_idx = nullptr,
                             const Trigger* trig = nullptr) {
    int rc = check_partial_args(geom, q, small, n_sel, full, tail_start, seq_lens, max_recent, out);
    if (rc != RK_OK) return rc;
    // What the step uses of the workspace lies at offsets that follow from the geometry alone; only the
    // partial outputs of the ticketed form grow with the launch (one slot per workgroup of a (sequence,
    // KV head), at most kMergeChunks): a bound on the rows decoded since the refresh that keeps growing
    // (the trigger's schedule) never outgrows a workspace sized for the context.
    if (!workspace || ((uintptr_t)workspace & 255u) != 0) return RK_ERR_WORKSPACE;
    Workspace ws = carve(geom, 1, 0, workspace);
    const size_t problems = (size_t)geom->batch * geom->n_kv_heads;
    const size_t before = (size_t)((char*)ws.part_o - (char*)workspace);
    const size_t slot = problems * (geom->n_q_heads / geom->n_kv_heads) * kD * sizeof(float);     // one partial output of every (sequence, KV head)
    if (workspace_bytes < before + slot) return RK_ERR_WORKSPACE;
    const size_t slots = (workspace_bytes - before) / slot;
    ws.max_chunks = slots < (size_t)kMergeChunks ? (int)slots : kMergeChunks;     // the launch takes no more workgroups than this
    return launch_partial(geom, q, small, n_sel, evict, full, tail_start, seq_lens, max_recent, out, pred, pred_val,
                          ws, stream, lazy_idx, trig);
}

extern "C" int rk_debug_set_slice_spin(int32_t spin) {
    if (spin < 0) return RK_ERR_INVALID_ARG;
    rk::g_slice_spin.store(spin, std::memory_order_relaxed);
    return RK_OK;
}

extern "C" int rk_partial_attn(const rk_geom* geom, const void* q, rk_kv small, int32_t n_sel,
                               rk_kv full, const int32_t* tail_start, const int32_t* seq_lens,
                               int32_t max_recent, void* out,
                               const int32_t* pred, int32_t pred_val,
                               void* workspace, size_t workspace_bytes, void* stream) {
    return partial_attn_impl(geom, q, small, n_sel, false, full, tail_start, seq_lens, max_recent, out, pred, pred_val,
                             workspace, workspace_bytes, stream);
}

extern "C" int rk_partial_attn_lazy(const rk_geom* geom, const void* q, rk_kv small, const int32_t* idx, int32_t k,
                                    int32_t fixed_size, rk_kv full, const int32_t* tail_start, const int32_t* seq_lens,
                                    int32_t max_recent, void* out,
                                    const int32_t* pred, int32_t pred_val,
                                    void* workspace, size_t workspace_bytes, void* stream) {
    if (!idx) return RK_ERR_INVALID_ARG;
    return partial_attn_impl(geom, q, small, k, fixed_size != 0, full, tail_start, seq_lens, max_recent, out,
                             pred, pred_val, workspace, workspace_bytes, stream, idx);
}

extern "C" int rk_partial_attn_fixed(const rk_geom* geom, const void* q, rk_kv small, int32_t k,
                                     rk_kv full, const int32_t* tail_start, const int32_t* seq_lens,
                                     int32_t max_recent, void* out,
                                     const int32_t* pred, int32_t pred_val,
                                     void* workspace, size_t workspace_bytes, void* stream) {
    return partial_attn_impl(geom, q, small, k, true, full, tail_start, seq_lens, max_recent, out, pred, pred_val,
                             workspace, workspace_bytes, stream);
}
extern "C" int rk_partial_attn_triggered(const rk_geom* geom, const void* q, rk_kv small, int32_t n_sel,
                                         int32_t fixed_size, rk_kv full, const int32_t* tail_start,
                                         const int32_t* seq_lens, int32_t max_recent, void* out,
                                         float* q_ref, float threshold, float* sim, int32_t* need_full,
                                         void* workspace, size_t workspace_bytes, void* stream) {
    if (!q_ref || !sim || !need_full || !aligned16(q_ref)) return RK_ERR_INVALID_ARG;
    const Trigger trig{q_ref, threshold, sim, need_full};
    return partial_attn_impl(geom, q, small, n_sel, fixed_size != 0, full, tail_start, seq_lens, max_recent, out,
                             nullptr, 0, workspace, workspace_bytes, stream, nullptr, &trig);
}

// ---- rk_partial_attn_static: the partial step for callers that cannot allocate ----
// The scratch memory of the step (arrival counters, per-workgroup statistics and partial outputs)
// lives in a file-scope device array instead of a caller's workspace.  Every GPU the library is
// loaded on holds its own copy of the array at its own address; that address is looked up once per
// device (hipGetSymbolAddress) and only the looked-up pointer is ever handed to kernels: in host
// code the array's name is a stand-in, not a device address.
namespace rk {
constexpr size_t kStaticScratchBytes = (size_t)RK_STATIC_SCRATCH_BYTES;
constexpr int kStaticMaxProblems = 4096;          // (sequence, KV head) pairs: one arrival counter line each
constexpr int kStaticMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static std::mutex g_static_mutex;
static unsigned char* g_static_ptr[kStaticMaxDevices];     // per device: its copy of `scratch`, counters cleared

__global__ void static_clear_kernel(int32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// The scratch of the current device.  First use on a device: the address is looked up and the
// counters are cleared by a small fill kernel on `stream` (not a memset: the call may be under
// graph capture), ahead of the step that is enqueued next on the same stream.
static int static_scratch(hipStream_t stream, unsigned char** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return RK_ERR_HIP;
    if (dev < 0 || dev >= kStaticMaxDevices) return RK_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (g_static_ptr[dev] == nullptr) {
        unsigned char* ptr = nullptr;
        if (hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return RK_ERR_HIP;
        if (((uintptr_t)ptr & 255u) != 0) return RK_ERR_HIP;
        hipLaunchKernelGGL(static_clear_kernel, dim3(kStaticMaxProblems * kCounterStride / 256), dim3(256), 0, stream,
                           (int32_t*)ptr, kStaticMaxProblems * kCounterStride);
        if (launch_status() != RK_OK) return RK_ERR_HIP;
        g_static_ptr[dev] = ptr;
    }
    *out = g_static_ptr[dev];
    return RK_OK;
}

// Fixed layout of the array, whatever the geometry: counters first (always kStaticMaxProblems of
// them, so a call with another geometry finds them where the last call left them: zero), then the
// regions whose size follows the call.  Returns the bytes used.
static size_t carve_static(const rk_geom* g, int32_t n_sel, int32_t max_recent, unsigned char* base, Workspace* w) {
    const size_t problems = (size_t)g->batch * g->n_kv_heads;
    const size_t G = (size_t)(g->n_q_heads / g->n_kv_heads);
    *w = Workspace{};
    w->max_chunks = merged_split_workgroups(n_sel, max_recent, (int64_t)problems, true);     // the launch's own count (ticketed merge)
    size_t off = 0;
    w->counters = (int32_t*)(base + off); off += (size_t)kStaticMaxProblems * kCounterStride * sizeof(int32_t);
    w->lse = (float*)(base + off);        off += align_up((size_t)g->batch * g->n_q_heads * sizeof(float), 256);
    w->part_ml = (float*)(base + off);    off += align_up(problems * kMaxChunks * G * 2 * sizeof(float), 256);
    w->part_o = (float*)(base + off);     off += align_up(problems * (size_t)w->max_chunks * G * kD * sizeof(float), 256);
    w->total = off;
    return off;
}
}  // namespace rk

extern "C" size_t rk_partial_attn_static_bytes(const rk_geom* geom, int32_t n_sel, int32_t max_recent) {
    if (check_geom(geom) != RK_OK || n_sel < 0 || max_recent < 0 || n_sel + (int64_t)max_recent <= 0 ||
        n_sel + (int64_t)max_recent > INT32_MAX) return 0;
    Workspace w;
    return carve_static(geom, n_sel, max_recent, nullptr, &w);
}

extern "C" int rk_partial_attn_static(const rk_geom* geom, const void* q, rk_kv small, int32_t n_sel,
                                      rk_kv full, const int32_t* tail_start, const int32_t* seq_lens,
                                      int32_t max_recent, void* out,
                                      const int32_t* pred, int32_t pred_val, void* stream) {
    int rc = check_partial_args(geom, q, small, n_sel, full, tail_start, seq_lens, max_recent, out);
    if (rc != RK_OK) return rc;
    if ((int64_t)geom->batch * geom->n_kv_heads > kStaticMaxProblems) return RK_ERR_STATIC_SCRATCH;
    Workspace ws;
    if (carve_static(geom, n_sel, max_recent, nullptr, &ws) > kStaticScratchBytes) return RK_ERR_STATIC_SCRATCH;
    unsigned char* base = nullptr;
    if ((rc = static_scratch((hipStream_t)stream, &base)) != RK_OK) return rc;
    carve_static(geom, n_sel, max_recent, base, &ws);
    return launch_partial(geom, q, small, n_sel, false, full, tail_start, seq_lens, max_recent, out, pred, pred_val,
                          ws, stream);
}
