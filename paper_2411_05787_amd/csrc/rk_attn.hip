// Split-K decode attention for gfx950: rk_full_attn and rk_partial_attn.
//
// One workgroup reduces a chunk of KV rows of one (sequence, KV head) for all G query heads
// of the GQA group, so every K/V byte is read from HBM once.  The workgroup that arrives
// last for a (sequence, KV head) merges the partial results and writes the output.
//
// Hand-over between workgroups (which may sit on different XCDs, each with its own L2):
// partial results are written with agent-scope atomic stores and read with agent-scope atomic
// loads, i.e. write-through / coherent accesses; a writer waits until its stores are
// acknowledged (s_waitcnt vmcnt(0)) before it takes its arrival ticket with an agent-scope
// atomic add.  No cache-wide release/acquire fence is used: on this chip one such fence per
// workgroup writes back and invalidates a whole L2 and costs more than the attention itself.
//
// Data path per wavefront and iteration (ROWS = 16 * TILES rows):
//   K rows  -> registers in MFMA operand layout (16-byte loads, no LDS)
//   S = Q K^T on the matrix cores: v_mfma_f32_16x16x32_bf16, M = query heads (padded to 16),
//             N = 16 rows, contraction over head_dim in 4 steps
//   softmax bookkeeping (running max / sum) on the lanes that hold S
//   P crosses to the V layout through LDS; raw scores (when weights are returned) are stored
//             straight from the S layout
//   O += P V on the vector ALU: each lane owns 8 consecutive dims of one row in four,
//             V rows loaded with fully coalesced 16-byte loads
// The K and V registers are double-buffered: the loads of a wavefront's next tile are issued
// before the current tile is computed.
#include "rk_internal.h"
#include "rk_device.h"

namespace rk {

struct AttnParams {
    const uint16_t* q;                 // bf16 [B, Hq, 128]
    const uint16_t* k1; const uint16_t* v1; int64_t s1_b, s1_h;   // small cache (TWO_SEG only)
    const uint16_t* k2; const uint16_t* v2; int64_t s2_b, s2_h;   // full cache
    const int32_t* tail_start;         // TWO_SEG only
    const int32_t* seq_lens;
    int32_t n_sel;                     // rows taken from the small cache (TWO_SEG only)
    int32_t max_rows2;                 // host bound on the rows taken from the full cache
    int32_t cap1, cap2;                // rows allocated in the small / full cache
    int32_t chunk;                     // rows per workgroup
    int32_t Hq, Hkv;
    float scale;
    uint16_t* out;                     // bf16 [B, Hq, 128]
    float* weights; int64_t w_stride;  // raw scores go here first (EMIT only)
    float* lse;                        // fp32 [B, Hq], never NULL here
    const int32_t* pred; int32_t pred_val;
    int32_t* counters; float* part_ml; float* part_o; int32_t max_chunks;
};

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
template <int G, int NW>
__device__ void merge_partials(const AttnParams& p, int b, int g, int nchunks, float* sW, float* sLc,
                               float* sM, double* sL) {
    constexpr int NT = NW * 64;
    constexpr int PER = G * kD / 2;               // pairs of consecutive dims to produce
    constexpr int ROUNDS = (PER + NT - 1) / NT;   // per thread: 1 (G <= 4) or 2
    constexpr int SUB = 16;                       // loads are issued in uniform groups of 16 chunks
    static_assert(kMergeChunks % SUB == 0, "chunk groups");
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t bg = (int64_t)b * p.Hkv + g;
    const float* ml = p.part_ml + bg * kMaxChunks * G * 2;
    const float* po = p.part_o + bg * p.max_chunks * G * kD;
    const int n_ml = nchunks * G;

    // Everything that has to come from memory is requested up front, in one round trip:
    // the (max, sum) pairs of every chunk and head, and this thread's slice of every partial output.
    uint64_t vml[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) vml[u] = coherent_load2(ml + (int64_t)min(u * NT + tid, n_ml - 1) * 2);
    uint64_t v[kMergeChunks];
    auto request = [&](int r) {
        const int e2 = min(r * NT + tid, PER - 1);
#pragma unroll
        for (int c0 = 0; c0 < kMergeChunks; c0 += SUB) {
            if (c0 < nchunks) {                   // uniform over the workgroup
#pragma unroll
                for (int u = 0; u < SUB; ++u)
                    v[c0 + u] = coherent_load2(po + (int64_t)min(c0 + u, nchunks - 1) * G * kD + 2 * e2);
            } else {
#pragma unroll
                for (int u = 0; u < SUB; ++u) v[c0 + u] = 0;
            }
        }
    };
    request(0);
    static_assert(4 * NT >= kMergeChunks * RK_MAX_GROUP || NW < 4, "one batch covers all (chunk, head) pairs");
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = u * NT + tid;
        if (i < n_ml) { sW[i] = lo_f(vml[u]); sLc[i] = hi_f(vml[u]); }
    }
    __syncthreads();
    // one wavefront per head: M = max_c m_c, w_c = e^{m_c - M} (overwrites m_c), L = sum_c w_c l_c
    for (int gi = w; gi < G; gi += NW) {
        float mx = -INFINITY;
        for (int c = lane; c < nchunks; c += 64) mx = fmaxf(mx, sW[c * G + gi]);
        mx = wave_max(mx);
        double ls = 0.0;                          // the sum that normalises the output: fp64
        for (int c = lane; c < nchunks; c += 64) {
            const float mc = sW[c * G + gi];
            const float wgt = (mc == -INFINITY) ? 0.f : fast_exp2((mc - mx) * kLog2e);
            sW[c * G + gi] = wgt;
            ls += (double)wgt * (double)sLc[c * G + gi];
        }
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) ls += __shfl_xor(ls, m);
        if (lane == 0) { sM[gi] = mx; sL[gi] = ls; }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
        if (r > 0) request(r);                    // G > 4: a second round trip for the other half
        const int e2 = r * NT + tid;
        if (e2 < PER) {
            const int gi = (2 * e2) / kD;
            float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
            for (int c = 0; c < kMergeChunks; ++c) {
                const float wgt = (c < nchunks) ? sW[c * G + gi] : 0.f;
                acc0 = fmaf(wgt, lo_f(v[c]), acc0);
                acc1 = fmaf(wgt, hi_f(v[c]), acc1);
            }
            const float L = (float)sL[gi];
            const float inv = L > 0.f ? 1.f / L : 0.f;
            const uint32_t packed = (uint32_t)f32_to_bf16(acc0 * inv) | ((uint32_t)f32_to_bf16(acc1 * inv) << 16);
            reinterpret_cast<uint32_t*>(p.out + ((int64_t)b * p.Hq + g * G) * kD)[e2] = packed;
        }
    }
    if (tid < G) {
        const double L = sL[tid];
        p.lse[(int64_t)b * p.Hq + g * G + tid] = L > 0.0 ? (float)((double)sM[tid] + log(L)) : -INFINITY;
    }
}

// Two wavefronts per SIMD (<= 256 registers each) whenever the accumulators leave room for it.
template <int G, int NW, int TILES, bool EMIT, bool TWO_SEG>
__global__ __launch_bounds__(NW * 64, (G <= 4 || TILES == 1) ? 2 : 1)
void attn_split_kernel(const AttnParams p) {
    constexpr int GP = (G + 3) / 4 * 4;      // heads padded to whole MFMA accumulator registers
    constexpr int NC = GP / 4;               // 16-lane groups whose accumulators hold real heads
    constexpr int ROWS = TILES * 16;         // rows per wavefront per iteration
    constexpr int NV = ROWS / 4;             // V loads per lane per iteration
    constexpr int RG = (G <= 4) ? 4 : 2;     // row groups of a wavefront kept apart in LDS
    constexpr int NT = NW * 64;

    const int c = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    if (p.pred != nullptr && p.pred[b] != p.pred_val) return;

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n16 = lane & 15, c4 = lane >> 4;     // S layout: row n16, heads 4*c4 .. 4*c4+3
    const int db = lane & 15, rg = lane >> 4;      // V layout: dims 8*db .. 8*db+7, rows = rg mod 4

    // ---- K rows of the first tile are requested before any length is known ----
    // Rows below `spec_rows` exist whatever the device-side lengths say (small cache: the first
    // n_sel rows; full cache: its capacity), so a chunk that lies wholly below it may be read
    // at once; rows that turn out to be past the end are masked like any other.  This takes the
    // round trip for seq_lens / tail_start off the critical path of every workgroup.
    const int r_first = c * p.chunk + w * ROWS;
    const int spec_rows = TWO_SEG ? min(p.n_sel, p.cap1) : p.cap2;
    const bool spec = (int64_t)(c + 1) * p.chunk <= spec_rows;
    uint4 kA[TILES][4], vA[NV], kB[TILES][4], vB[NV];
    if (spec) {
        const uint16_t* kspec = (TWO_SEG ? p.k1 + (int64_t)b * p.s1_b + (int64_t)g * p.s1_h
                                         : p.k2 + (int64_t)b * p.s2_b + (int64_t)g * p.s2_h) + c4 * 8;
#pragma unroll
        for (int t = 0; t < TILES; ++t)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                kA[t][kk] = *reinterpret_cast<const uint4*>(kspec + (int64_t)(r_first + t * 16 + n16) * kD + kk * 32);
    }

    // ---- the row list of this (sequence, KV head) ----
    // (device-side lengths are clamped to the allocated rows: no access leaves the caches)
    const int len = min(p.seq_lens[b], p.cap2);
    int n1 = 0, start2 = 0;
    if (TWO_SEG) {
        const int t0 = min(max(p.tail_start[b], 0), p.cap2);
        n1 = min(min(p.n_sel, t0), p.cap1);
        n1 = max(n1, 0);
        start2 = t0;
    }
    const int n2 = min(max(len - start2, 0), p.max_rows2);
    const int n = n1 + n2;
    const int nchunks = max(1, (n + p.chunk - 1) / p.chunk);
    if (c >= nchunks) return;
    const int row0 = c * p.chunk;
    const int row1 = min(n, row0 + p.chunk);

    const uint16_t* kb1 = nullptr; const uint16_t* vb1 = nullptr;
    if (TWO_SEG) {
        kb1 = p.k1 + (int64_t)b * p.s1_b + (int64_t)g * p.s1_h;
        vb1 = p.v1 + (int64_t)b * p.s1_b + (int64_t)g * p.s1_h;
    }
    // row r of the list lives at base2 + (start2 + r - n1) * 128 once r >= n1
    const uint16_t* kb2 = p.k2 + (int64_t)b * p.s2_b + (int64_t)g * p.s2_h + (int64_t)(start2 - n1) * kD;
    const uint16_t* vb2 = p.v2 + (int64_t)b * p.s2_b + (int64_t)g * p.s2_h + (int64_t)(start2 - n1) * kD;

    __shared__ __attribute__((aligned(16))) float sP[NW][ROWS][GP];
    __shared__ __attribute__((aligned(16))) float sAlpha[NW][GP];
    __shared__ __attribute__((aligned(16))) float sMw[NW][GP];
    __shared__ __attribute__((aligned(16))) float sLw[NW][GP];
    __shared__ __attribute__((aligned(16))) float sO[NW * RG][G][kD];   // reused by the merge
    __shared__ float sMf[GP];
    __shared__ double sLf[GP];
    __shared__ int sTicket;
    static_assert(NW * RG * G * kD >= 2 * kMergeChunks * G, "merge scratch must fit in the output staging buffer");

    // ---- Q as the A operand: lane (n16, c4) holds head n16, dims 8*(4*kk + c4) .. +7 ----
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

    float m_run[4], l_run[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { m_run[i] = -INFINITY; l_run[i] = 0.f; }
    float o[G][8];
#pragma unroll
    for (int gi = 0; gi < G; ++gi)
#pragma unroll
        for (int e = 0; e < 8; ++e) o[gi][e] = 0.f;

    // ---- loads: rows past the end of the chunk re-read its last row (masked later) ----
    auto load_k = [&](uint4 (&kreg)[TILES][4], int r) {
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            const int row = min(r + t * 16 + n16, row1 - 1);
            const uint16_t* base = (TWO_SEG && row < n1) ? kb1 : kb2;
            const uint16_t* rp = base + (int64_t)row * kD + c4 * 8;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) kreg[t][kk] = *reinterpret_cast<const uint4*>(rp + kk * 32);
        }
    };
    auto load_v = [&](uint4 (&vreg)[NV], int r) {
#pragma unroll
        for (int jj = 0; jj < NV; ++jj) {
            const int row = min(r + jj * 4 + rg, row1 - 1);
            const uint16_t* base = (TWO_SEG && row < n1) ? vb1 : vb2;
            vreg[jj] = *reinterpret_cast<const uint4*>(base + (int64_t)row * kD + db * 8);
        }
    };
    auto compute_tile = [&](uint4 (&kreg)[TILES][4], uint4 (&vreg)[NV], int r) {
        // ---- S = Q K^T: lane (n16, c4) gets heads 4*c4+i of row r + 16 t + n16 ----
        float s[TILES][4];
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[kk], __builtin_bit_cast(bf16x8, kreg[t][kk]),
                                                              acc, 0, 0, 0);
            const bool valid = (r + t * 16 + n16) < row1;
#pragma unroll
            for (int i = 0; i < 4; ++i) s[t][i] = valid ? acc[i] * p.scale : -INFINITY;
        }

        // ---- raw scores out, straight from the lanes that hold them: 16 consecutive rows of one
        //      head are a 64-byte segment ----
        if (EMIT) {
            if (c4 < NC) {
                float* wrow = p.weights + ((int64_t)b * p.Hq + (int64_t)g * G + c4 * 4) * p.w_stride + r + n16;
#pragma unroll
                for (int t = 0; t < TILES; ++t) {
                    if (r + t * 16 + n16 < row1) {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (c4 * 4 + i < G) wrow[(int64_t)i * p.w_stride + t * 16] = s[t][i];
                    }
                }
            }
        }

        // ---- running softmax statistics of this wavefront ----
        float alpha[4], pr[TILES][4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float mx = s[0][i];
#pragma unroll
            for (int t = 1; t < TILES; ++t) mx = fmaxf(mx, s[t][i]);
            mx = row16_max(mx);
            const float m_new = fmaxf(m_run[i], mx);       // finite: row r is always valid
            alpha[i] = fast_exp2((m_run[i] - m_new) * kLog2e);
            m_run[i] = m_new;
            float ps = 0.f;
#pragma unroll
            for (int t = 0; t < TILES; ++t) {
                pr[t][i] = fast_exp2((s[t][i] - m_new) * kLog2e);
                ps += pr[t][i];
            }
            l_run[i] = l_run[i] * alpha[i] + ps;            // per-lane share, summed at the end
        }
        if (c4 < NC) {
#pragma unroll
            for (int t = 0; t < TILES; ++t) {
                *reinterpret_cast<float4*>(&sP[w][t * 16 + n16][c4 * 4]) =
                    make_float4(pr[t][0], pr[t][1], pr[t][2], pr[t][3]);
            }
            if (n16 == 0)
                *reinterpret_cast<float4*>(&sAlpha[w][c4 * 4]) = make_float4(alpha[0], alpha[1], alpha[2], alpha[3]);
        }
        wave_lds_sync();

        // ---- O = alpha O + P V ----
        {
            float al[GP];
#pragma unroll
            for (int q4 = 0; q4 < NC; ++q4) {
                const float4 t4 = *reinterpret_cast<const float4*>(&sAlpha[w][q4 * 4]);
                al[q4 * 4 + 0] = t4.x; al[q4 * 4 + 1] = t4.y; al[q4 * 4 + 2] = t4.z; al[q4 * 4 + 3] = t4.w;
            }
#pragma unroll
            for (int gi = 0; gi < G; ++gi)
#pragma unroll
                for (int e = 0; e < 8; ++e) o[gi][e] *= al[gi];
        }
#pragma unroll
        for (int jj = 0; jj < NV; ++jj) {
            float pv[GP];
#pragma unroll
            for (int q4 = 0; q4 < NC; ++q4) {
                const float4 t4 = *reinterpret_cast<const float4*>(&sP[w][jj * 4 + rg][q4 * 4]);
                pv[q4 * 4 + 0] = t4.x; pv[q4 * 4 + 1] = t4.y; pv[q4 * 4 + 2] = t4.z; pv[q4 * 4 + 3] = t4.w;
            }
            const uint4 u = vreg[jj];
            const float vf[8] = {bf16_lo(u.x), bf16_hi(u.x), bf16_lo(u.y), bf16_hi(u.y),
                                 bf16_lo(u.z), bf16_hi(u.z), bf16_lo(u.w), bf16_hi(u.w)};
#pragma unroll
            for (int gi = 0; gi < G; ++gi)
#pragma unroll
                for (int e = 0; e < 8; ++e) o[gi][e] = fmaf(pv[gi], vf[e], o[gi][e]);
        }
        wave_lds_sync();      // sP / sAlpha are rewritten by the next tile
    };

    // Two register buffers: the loads of the next tile are in flight while this one is computed,
    // so a wavefront never stops requesting memory while it has rows left.
    {
        const int step = NW * ROWS;
        int r = r_first;
        if (r < row1) {
            // the early request stands unless part of this chunk maps to the tail of the full cache
            const bool spec_ok = spec && (!TWO_SEG || (c + 1) * p.chunk <= n1);
            if (!spec_ok) load_k(kA, r);
            load_v(vA, r);
        }
        while (r < row1) {
            const int rn = r + step;
            if (rn < row1) { load_k(kB, rn); load_v(vB, rn); }
            compute_tile(kA, vA, r);
            if (rn >= row1) break;
            const int rnn = rn + step;
            if (rnn < row1) { load_k(kA, rnn); load_v(vA, rnn); }
            compute_tile(kB, vB, rn);
            r = rnn;
        }
    }

    // ---- wavefront results to LDS ----
#pragma unroll
    for (int i = 0; i < 4; ++i) l_run[i] = row16_sum(l_run[i]);
    if (c4 < NC && n16 == 0) {
        *reinterpret_cast<float4*>(&sMw[w][c4 * 4]) = make_float4(m_run[0], m_run[1], m_run[2], m_run[3]);
        *reinterpret_cast<float4*>(&sLw[w][c4 * 4]) = make_float4(l_run[0], l_run[1], l_run[2], l_run[3]);
    }
    if (RG == 2) {
#pragma unroll
        for (int gi = 0; gi < G; ++gi)
#pragma unroll
            for (int e = 0; e < 8; ++e) o[gi][e] += __shfl_xor(o[gi][e], 32);
    }
    if (rg < RG) {
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            float4* dst = reinterpret_cast<float4*>(&sO[w * RG + rg][gi][db * 8]);
            dst[0] = make_float4(o[gi][0], o[gi][1], o[gi][2], o[gi][3]);
            dst[1] = make_float4(o[gi][4], o[gi][5], o[gi][6], o[gi][7]);
        }
    }
    __syncthreads();

    // ---- merge the NW wavefronts and publish the partial result of this chunk ----
    const int64_t bg = (int64_t)b * p.Hkv + g;
    float* ml = p.part_ml + (bg * kMaxChunks + c) * G * 2;
    float* po = p.part_o + (bg * p.max_chunks + c) * G * kD;
    for (int e2 = tid; e2 < G * kD / 2; e2 += NT) {           // two consecutive dims per thread
        const int gi = (2 * e2) / kD, d = (2 * e2) % kD;
        float M = sMw[0][gi];
#pragma unroll
        for (int ww = 1; ww < NW; ++ww) M = fmaxf(M, sMw[ww][gi]);
        float acc0 = 0.f, acc1 = 0.f, L = 0.f;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) {
            const float mw = sMw[ww][gi];
            const float sc = (mw == -INFINITY) ? 0.f : fast_exp2((mw - M) * kLog2e);
            float p0 = 0.f, p1 = 0.f;
#pragma unroll
            for (int rr = 0; rr < RG; ++rr) {
                const float2 t2 = *reinterpret_cast<const float2*>(&sO[ww * RG + rr][gi][d]);
                p0 += t2.x; p1 += t2.y;
            }
            acc0 = fmaf(sc, p0, acc0);
            acc1 = fmaf(sc, p1, acc1);
            L = fmaf(sc, sLw[ww][gi], L);
        }
        if (EMIT) {       // merged by the next kernel: ordinary stores
            *reinterpret_cast<float2*>(po + 2 * e2) = make_float2(acc0, acc1);
            if (d == 0) *reinterpret_cast<float2*>(ml + gi * 2) = make_float2(M, L);
        } else {
            coherent_store2(po + 2 * e2, acc0, acc1);
            if (d == 0) coherent_store2(ml + gi * 2, M, L);
        }
    }
    if (EMIT) return;

    // ---- the workgroup that arrives last for (b, g) merges all chunks ----
    wait_stores_acknowledged();
    __syncthreads();
    if (tid == 0) sTicket = __hip_atomic_fetch_add(&p.counters[bg], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (sTicket != nchunks - 1) return;
    merge_partials<G, NW>(p, b, g, nchunks, &sO[0][0][0], &sO[0][0][0] + kMergeChunks * G, sMf, sLf);
    if (tid == 0) __hip_atomic_store(&p.counters[bg], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // next call
}

// Second kernel of a full step that returns the attention weights.  Every workgroup first
// rebuilds lse of its (sequence, query head) from the per-chunk (max, sum) pairs, in fp64.
// Workgroup x = 0 then merges the partial outputs of that head; workgroups x >= 1 turn
// kNormTile raw scores each into weights[b,h,j] = exp(s[b,h,j] - lse[b,h]), in place.  The
// exponent is formed as an exact fp32 pair (two-sum) minus the low part of lse, so a weight
// carries the error of its score and of expf only (a plain fp32 subtraction alone would cost
// up to 5e-7 relative, which is the size of the gaps that decide the selection).
constexpr int kNormTile = 4096;

__global__ __launch_bounds__(256)
void merge_normalise_kernel(const AttnParams p, int G) {
    const int x = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    if (p.pred != nullptr && p.pred[b] != p.pred_val) return;
    const int tid = threadIdx.x;
    const int g = h / G, gi = h % G;
    const int len = min(max(min(p.seq_lens[b], p.cap2), 0), p.max_rows2);
    const int nchunks = max(1, (len + p.chunk - 1) / p.chunk);
    const int j0 = (x - 1) * kNormTile;
    if (x >= 1 && j0 >= len) return;

    __shared__ __attribute__((aligned(8))) float sRed[8];
    __shared__ float sW[kMaxChunks];
    __shared__ float sLse[2];
    __shared__ double sL64;
    __shared__ float sAcc[4][kD];
    constexpr int PER = kNormTile / 256;         // scores per thread
    constexpr int BATCH = 16;                    // partial outputs per thread and round trip

    const int64_t bg = (int64_t)b * p.Hkv + g;
    const float* ml = p.part_ml + (bg * kMaxChunks * G + gi) * 2;
    float* row = p.weights + ((int64_t)b * p.Hq + h) * p.w_stride;
    const int cg = tid >> 6, d2 = tid & 63;
    const float* po = p.part_o + (bg * p.max_chunks * G + gi) * kD + 2 * d2;

    // ---- request everything this workgroup needs before the first wait ----
    float m = -INFINITY, l = 0.f;
    if (tid < nchunks) {                                   // nchunks <= kMaxChunks == blockDim
        const float2 t2 = *reinterpret_cast<const float2*>(ml + (int64_t)tid * G * 2);
        m = t2.x; l = t2.y;
    }
    float sc[PER];
    float2 v[BATCH];
    if (x >= 1) {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int j = j0 + i * 256 + tid;
            sc[i] = (j < len) ? row[j] : 0.f;
        }
    } else {
#pragma unroll
        for (int u = 0; u < BATCH; ++u) v[u] = *reinterpret_cast<const float2*>(po + (int64_t)min(cg + 4 * u, nchunks - 1) * G * kD);
    }

    // ---- lse of (b, h) in fp64 ----
    const float M = block_max<4>(m, sRed);
    const float wgt = (m == -INFINITY) ? 0.f : fast_exp2((m - M) * kLog2e);
    if (tid < nchunks) sW[tid] = wgt;
    const double L64 = block_sum_f64<4>((double)wgt * (double)l, reinterpret_cast<double*>(sRed));
    if (tid == 0) {
        float hi = -INFINITY, lo = 0.f;
        if (L64 > 0.0) {
            const double l64 = (double)M + log(L64);
            hi = (float)l64;
            lo = (float)(l64 - (double)hi);
        }
        sLse[0] = hi; sLse[1] = lo; sL64 = L64;
    }
    __syncthreads();

    if (x == 0) {
        // out[b,h,:] = sum_c w_c o_c[h,:] / L: four groups of 64 lanes take every fourth chunk
        float acc0 = 0.f, acc1 = 0.f;
        for (int c0 = cg; c0 < nchunks; c0 += 4 * BATCH) {
            if (c0 != cg) {
#pragma unroll
                for (int u = 0; u < BATCH; ++u)
                    v[u] = *reinterpret_cast<const float2*>(po + (int64_t)min(c0 + 4 * u, nchunks - 1) * G * kD);
            }
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const float wc = (c0 + 4 * u < nchunks) ? sW[c0 + 4 * u] : 0.f;
                acc0 = fmaf(wc, v[u].x, acc0);
                acc1 = fmaf(wc, v[u].y, acc1);
            }
        }
        sAcc[cg][2 * d2] = acc0; sAcc[cg][2 * d2 + 1] = acc1;
        __syncthreads();
        if (tid < kD) {
            const float L = (float)sL64;
            const float o = L > 0.f ? (sAcc[0][tid] + sAcc[1][tid] + sAcc[2][tid] + sAcc[3][tid]) / L : 0.f;
            p.out[((int64_t)b * p.Hq + h) * kD + tid] = f32_to_bf16(o);
        }
        if (tid == 0) p.lse[(int64_t)b * p.Hq + h] = sLse[0];
        return;
    }

    const float nl = -sLse[0], ll = sLse[1];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int j = j0 + i * 256 + tid;
        if (j < len) {
            const float s = sc[i];
            const float hi = s + nl;
            const float bp = hi - s;
            const float lo = (s - (hi - bp)) + (nl - bp) - ll;     // s - lse = hi + lo, |lo| << 1
            const float e = expf(hi);
            row[j] = fmaf(e, lo, e);
        }
    }
}

template <int G, bool EMIT, bool TWO_SEG>
static int launch_split_g(const AttnParams& p, int batch, int nchunk_grid, hipStream_t st) {
    dim3 grid(nchunk_grid, p.Hkv, batch);
#ifndef RK_BIG_TILES
#define RK_BIG_TILES 2
#endif
    if (p.chunk >= 128) {       // 32 rows per wavefront and tile (16 for the larger groups, whose
                                // accumulators take the registers); >= 2 tiles per wavefront from chunk 256 up
        hipLaunchKernelGGL((attn_split_kernel<G, 4, (G <= 4 ? RK_BIG_TILES : 1), EMIT, TWO_SEG>), grid, dim3(256), 0, st, p);
    } else {
        hipLaunchKernelGGL((attn_split_kernel<G, 4, 1, EMIT, TWO_SEG>), grid, dim3(256), 0, st, p);
    }
    return launch_status();
}

template <bool EMIT, bool TWO_SEG>
static int launch_split(const AttnParams& p, int batch, int G, int nchunk_grid, hipStream_t st) {
    switch (G) {
        case 1: return launch_split_g<1, EMIT, TWO_SEG>(p, batch, nchunk_grid, st);
        case 2: return launch_split_g<2, EMIT, TWO_SEG>(p, batch, nchunk_grid, st);
        case 3: return launch_split_g<3, EMIT, TWO_SEG>(p, batch, nchunk_grid, st);
        case 4: return launch_split_g<4, EMIT, TWO_SEG>(p, batch, nchunk_grid, st);
        case 5: return launch_split_g<5, EMIT, TWO_SEG>(p, batch, nchunk_grid, st);
        case 6: return launch_split_g<6, EMIT, TWO_SEG>(p, batch, nchunk_grid, st);
        case 7: return launch_split_g<7, EMIT, TWO_SEG>(p, batch, nchunk_grid, st);
        case 8: return launch_split_g<8, EMIT, TWO_SEG>(p, batch, nchunk_grid, st);
        default: return RK_ERR_UNSUPPORTED;
    }
}

}  // namespace rk

using namespace rk;

static int full_attn_impl(const rk_geom* geom, const void* q, rk_kv full,
                          const int32_t* seq_lens, int32_t max_len,
                          void* out, float* weights, int64_t w_stride, float* lse,
                          const int32_t* pred, int32_t pred_val,
                          void* workspace, size_t workspace_bytes, void* stream, bool scores_only) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!q || (!out && !scores_only) || !seq_lens || max_len <= 0) return RK_ERR_INVALID_ARG;
    if (!aligned16(q) || ((uintptr_t)out & 1u)) return RK_ERR_INVALID_ARG;
    if ((rc = check_kv(full)) != RK_OK) return rc;
    if (weights && (w_stride < max_len || ((uintptr_t)weights & 3u))) return RK_ERR_INVALID_ARG;
    Workspace ws;
    if ((rc = check_workspace(geom, max_len, 0, workspace, workspace_bytes, &ws)) != RK_OK) return rc;

    const int G = geom->n_q_heads / geom->n_kv_heads;
    AttnParams p{};
    p.q = (const uint16_t*)q;
    p.k2 = (const uint16_t*)full.k; p.v2 = (const uint16_t*)full.v;
    p.s2_b = full.stride_b; p.s2_h = full.stride_h;
    p.seq_lens = seq_lens;
    p.n_sel = 0;
    p.max_rows2 = max_len;
    p.cap1 = 0; p.cap2 = (int32_t)full.capacity;
    p.chunk = attn_chunk_rows(max_len, (int64_t)geom->batch * geom->n_kv_heads, weights ? kMaxChunks : kMergeChunks);
    p.Hq = geom->n_q_heads; p.Hkv = geom->n_kv_heads;
    p.scale = geom->scale;
    p.out = (uint16_t*)out;
    p.weights = weights; p.w_stride = w_stride;
    p.lse = lse ? lse : ws.lse;
    p.pred = pred; p.pred_val = pred_val;
    p.counters = ws.counters; p.part_ml = ws.part_ml; p.part_o = ws.part_o; p.max_chunks = ws.max_chunks;
    const int nchunk_grid = (max_len + p.chunk - 1) / p.chunk;
    hipStream_t st = (hipStream_t)stream;
    if (weights) {
        rc = launch_split<true, false>(p, geom->batch, G, nchunk_grid, st);
        if (rc != RK_OK || scores_only) return rc;
        dim3 grid(1 + (max_len + kNormTile - 1) / kNormTile, geom->n_q_heads, geom->batch);
        hipLaunchKernelGGL(merge_normalise_kernel, grid, dim3(256), 0, st, p, G);
        return launch_status();
    }
    return launch_split<false, false>(p, geom->batch, G, nchunk_grid, st);
}

extern "C" int rk_full_attn(const rk_geom* geom, const void* q, rk_kv full,
                            const int32_t* seq_lens, int32_t max_len,
                            void* out, float* weights, int64_t w_stride, float* lse,
                            const int32_t* pred, int32_t pred_val,
                            void* workspace, size_t workspace_bytes, void* stream) {
    return full_attn_impl(geom, q, full, seq_lens, max_len, out, weights, w_stride, lse, pred, pred_val,
                          workspace, workspace_bytes, stream, false);
}

extern "C" int rk_full_attn_scores(const rk_geom* geom, const void* q, rk_kv full,
                                   const int32_t* seq_lens, int32_t max_len,
                                   float* scores, int64_t s_stride,
                                   const int32_t* pred, int32_t pred_val,
                                   void* workspace, size_t workspace_bytes, void* stream) {
    if (!scores) return RK_ERR_INVALID_ARG;
    return full_attn_impl(geom, q, full, seq_lens, max_len, nullptr, scores, s_stride, nullptr, pred, pred_val,
                          workspace, workspace_bytes, stream, true);
}

extern "C" int rk_partial_attn(const rk_geom* geom, const void* q, rk_kv small, int32_t n_sel,
                               rk_kv full, const int32_t* tail_start, const int32_t* seq_lens,
                               int32_t max_recent, void* out,
                               const int32_t* pred, int32_t pred_val,
                               void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!q || !out || !seq_lens || !tail_start || n_sel < 0 || max_recent < 0) return RK_ERR_INVALID_ARG;
    if (n_sel + (int64_t)max_recent <= 0 || n_sel + (int64_t)max_recent > INT32_MAX) return RK_ERR_INVALID_ARG;
    if (!aligned16(q) || ((uintptr_t)out & 1u)) return RK_ERR_INVALID_ARG;
    if ((rc = check_kv(full)) != RK_OK) return rc;
    if (n_sel > 0 && (rc = check_kv(small)) != RK_OK) return rc;
    const int max_rows = n_sel + max_recent;
    Workspace ws;
    if ((rc = check_workspace(geom, max_rows, 0, workspace, workspace_bytes, &ws)) != RK_OK) return rc;

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
    p.max_rows2 = max_recent;
    p.cap1 = n_sel > 0 ? (int32_t)small.capacity : 0; p.cap2 = (int32_t)full.capacity;
    p.chunk = attn_chunk_rows(max_rows, (int64_t)geom->batch * geom->n_kv_heads, kMergeChunks);
    p.Hq = geom->n_q_heads; p.Hkv = geom->n_kv_heads;
    p.scale = geom->scale;
    p.out = (uint16_t*)out;
    p.lse = ws.lse;
    p.pred = pred; p.pred_val = pred_val;
    p.counters = ws.counters; p.part_ml = ws.part_ml; p.part_o = ws.part_o; p.max_chunks = ws.max_chunks;
    const int nchunk_grid = (max_rows + p.chunk - 1) / p.chunk;
    return launch_split<false, true>(p, geom->batch, G, nchunk_grid, (hipStream_t)stream);
}
