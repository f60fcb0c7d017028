// Prefill-side initialisation of the small cache from an observation window: rk_window_select.
//
// The W queries of the last prompt tokens vote for the rows of the full cache (Section 2.2
// "Prefilling stage": the scores of the last prompt token; Section 3 and Appendix A.1 "Baseline
// Settings": the last few tokens of the prompt, the observation window).  Per query head,
//   votes[j] = sum_i softmax_{j' <= p_i}(scale <q_i, k_j'>)[j],  p_i = len - W + i  (causal),
// then the selection of rk_topk_select runs on the votes.
//
// Only K is read, twice:
//   pass 1  window_lse_kernel     log-sum-exp of every (query, head) column, split over
//                                 workgroups like the decode kernels; window_lse_merge_kernel
//                                 folds the partial (max, sum) pairs
//   pass 2  window_vote_kernel    the same stream again: normalised scores, summed over the
//                                 window's queries on the lanes, stored once per (head, row)
// Storing the raw scores of every query instead (one pass) would write and re-read
// W * Hq * len * 4 bytes: more than the second pass over K from W = 8 on at the usual shapes.
//
// Per tile of 32 rows the scores of all columns come from the matrix cores
// (v_mfma_f32_16x16x32_bf16, K rows as the 16-row operand straight from global memory in
// operand layout; the queries, 16 columns at a time, from LDS).  Column c = i * Gp + gi: query
// i of the window, head gi of the GQA group, Gp = G rounded up to a power of two so that a lane
// keeps the same head in every block of 16 columns and the sum over the window is a per-lane
// sum over blocks plus log2(16 / Gp) cross-lane steps.
#include "rk_internal.h"
#include "rk_device.h"

namespace rk {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct WindowParams {
    const uint16_t* q;                 // bf16 [B, W, Hq, 128]
    const uint16_t* k; int64_t s_b, s_h; int32_t cap;
    const int32_t* seq_lens; int32_t max_rows;
    int32_t W, G, gp_shift;            // Gp = 1 << gp_shift
    int32_t ncb;                       // blocks of 16 columns
    int32_t nch, Hq, Hkv;
    float scale;
    float* part;                       // fp32 [B*Hkv][nch][ncb*16][2]  (max, sum) per workgroup and column
    float* lse;                        // fp32 [B*Hkv][ncb*16][2]       lse as hi + lo
    float* votes; int64_t v_stride; int32_t v_vec;
    const int32_t* pred; int32_t pred_val;
};

constexpr int kWinWaves = 4, kWinRows = 32;
constexpr int kQStride = kD + 8;       // bf16 elements between columns in LDS: 272 bytes, conflict-free 16-byte reads

__device__ __forceinline__ int window_workgroups(int n_rows, int nch) {
    return max(1, min(nch, (n_rows + kWinWaves * kWinRows - 1) / (kWinWaves * kWinRows)));
}

// Last row that column `col` may see (-1: the column does not exist).
__device__ __forceinline__ int column_limit(const WindowParams& p, int col, int n) {
    const int i = col >> p.gp_shift, gi = col & ((1 << p.gp_shift) - 1);
    const int pos = n - p.W + i;
    return (i < p.W && gi < p.G && pos >= 0) ? pos : -1;
}

// The window's queries of KV head g into LDS, one column per (query, head), zero where none.
__device__ __forceinline__ void stage_queries(const WindowParams& p, int b, int g, int n, int ncol, uint16_t* sQ) {
    for (int x = threadIdx.x; x < ncol * 16; x += blockDim.x) {
        const int col = x >> 4, piece = x & 15;
        uint4 u = make_uint4(0, 0, 0, 0);
        if (column_limit(p, col, n) >= 0) {
            const int i = col >> p.gp_shift, gi = col & ((1 << p.gp_shift) - 1);
            u = *reinterpret_cast<const uint4*>(p.q + (((int64_t)b * p.W + i) * p.Hq + (int64_t)g * p.G + gi) * kD + piece * 8);
        }
        *reinterpret_cast<uint4*>(sQ + col * kQStride + piece * 8) = u;
    }
}

// Rows r .. r + 31 of K in operand layout (rows past the end repeat the last row; masked later).
__device__ __forceinline__ void load_k_tile(u32x4 (&dst)[2][4], const uint16_t* kb, int r, int n16, int n) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int row = min(r + t * 16 + n16, n - 1);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            dst[t][kk] = *reinterpret_cast<const u32x4*>(kb + (int64_t)row * kD + kk * 32);
    }
}

// Scores of one tile against the 16 columns of block cb: s[t][i] is row r + 16 t + 4 c4 + i of
// column cb * 16 + n16, scaled, -inf beyond `limit`.
__device__ __forceinline__ void tile_scores(const u32x4 (&k)[2][4], const uint16_t* sQ, int cb, int n16, int c4,
                                            int r, int limit, float scale, float (&s)[2][4]) {
    bf16x8 qa[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        qa[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(sQ + (cb * 16 + n16) * kQStride + (kk * 4 + c4) * 8));
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k[t][kk]), qa[kk], acc, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) s[t][i] = (r + t * 16 + 4 * c4 + i <= limit) ? acc[i] * scale : -INFINITY;
    }
}

// (m, l) <- (m, l) merged with (m2, l2): running max and sum of exponentials relative to it.
__device__ __forceinline__ void merge_ml(float& m, float& l, float m2, float l2) {
    const float M = fmaxf(m, m2);
    const float a = (m == -INFINITY) ? 0.f : fast_exp2((m - M) * kLog2e);
    const float c = (m2 == -INFINITY) ? 0.f : fast_exp2((m2 - M) * kLog2e);
    l = l * a + l2 * c;
    m = M;
}

extern __shared__ __attribute__((aligned(16))) unsigned char window_lds[];

// Pass 1.  The running (max, sum) of a lane's column in every block lives in LDS (one float2 per
// lane and block), so that the number of blocks is a run-time value and the register count does
// not grow with the window.
__global__ __launch_bounds__(kWinWaves * 64)
void window_lse_kernel(const WindowParams p) {
    constexpr int NW = kWinWaves, NT = kWinWaves * 64;
    const int ncb = p.ncb, ncol = ncb * 16;
    const int c = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    if (p.pred != nullptr && p.pred[b] != p.pred_val) return;
    const int n = min(max(min(p.seq_lens[b], p.cap), 0), p.max_rows);
    if (n == 0 || c >= window_workgroups(n, p.nch)) return;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n16 = lane & 15, c4 = lane >> 4;
    uint16_t* sQ = reinterpret_cast<uint16_t*>(window_lds);
    float2* sRun = reinterpret_cast<float2*>(window_lds + (size_t)ncol * kQStride * 2);   // [ncb][NT]
    float* sM = reinterpret_cast<float*>(sRun + (size_t)ncb * NT);                        // [NW][ncol]
    float* sL = sM + NW * ncol;
    stage_queries(p, b, g, n, ncol, sQ);
    for (int cb = 0; cb < ncb; ++cb) sRun[cb * NT + tid] = make_float2(-INFINITY, 0.f);
    __syncthreads();

    const uint16_t* kb = p.k + (int64_t)b * p.s_b + (int64_t)g * p.s_h + c4 * 8;
    const int step = p.nch * NW * kWinRows;
    u32x4 kA[2][4], kB[2][4];
    auto tile = [&](const u32x4 (&k)[2][4], int r) {
#pragma unroll 1
        for (int cb = 0; cb < ncb; ++cb) {
            float s[2][4];
            tile_scores(k, sQ, cb, n16, c4, r, column_limit(p, cb * 16 + n16, n), p.scale, s);
            const float mx = fmaxf(fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3])),
                                   fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3])));
            const float2 run = sRun[cb * NT + tid];
            const float m_new = fmaxf(run.x, mx);
            if (m_new != -INFINITY) {
                float ps = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) ps += fast_exp2((s[e >> 2][e & 3] - m_new) * kLog2e);
                sRun[cb * NT + tid] = make_float2(m_new, run.y * fast_exp2((run.x - m_new) * kLog2e) + ps);
            }
        }
    };
    int r = (c * NW + w) * kWinRows;
    if (r < n) load_k_tile(kA, kb, r, n16, n);
    if (r + step < n) load_k_tile(kB, kb, r + step, n16, n);
    while (r < n) {
        tile(kA, r);
        if (r + 2 * step < n) load_k_tile(kA, kb, r + 2 * step, n16, n);
        r += step;
        if (r >= n) break;
        tile(kB, r);
        if (r + 2 * step < n) load_k_tile(kB, kb, r + 2 * step, n16, n);
        r += step;
    }
    // fold the four row groups of the wavefront, then the wavefronts
    for (int cb = 0; cb < ncb; ++cb) {
        const float2 run = sRun[cb * NT + tid];
        float m = run.x, l = run.y;
#pragma unroll
        for (int x = 16; x < 64; x <<= 1) {
            const float m2 = __shfl_xor(m, x), l2 = __shfl_xor(l, x);
            merge_ml(m, l, m2, l2);
        }
        if (c4 == 0) { sM[w * ncol + cb * 16 + n16] = m; sL[w * ncol + cb * 16 + n16] = l; }
    }
    __syncthreads();
    const int64_t bg = (int64_t)b * p.Hkv + g;
    float* part = p.part + ((bg * p.nch + c) * ncol) * 2;
    for (int col = tid; col < ncol; col += NT) {
        float m = sM[col], l = sL[col];
#pragma unroll
        for (int ww = 1; ww < NW; ++ww) merge_ml(m, l, sM[ww * ncol + col], sL[ww * ncol + col]);
        *reinterpret_cast<float2*>(part + col * 2) = make_float2(m, l);
    }
}

// lse of every column from the per-workgroup pairs: one workgroup per (block of 16 columns,
// sequence, KV head); thread (n16, cl) folds the pairs of column n16 from workgroups cl, cl + 16,
// ...; thread (n16, 0) folds the 16 results.  Stored as hi + lo (two floats) so that scores
// normalised with it keep full fp32 precision.
__global__ __launch_bounds__(256)
void window_lse_merge_kernel(const WindowParams p) {
    const int cb = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    if (p.pred != nullptr && p.pred[b] != p.pred_val) return;
    const int n = min(max(min(p.seq_lens[b], p.cap), 0), p.max_rows);
    if (n == 0) return;
    const int nchunks = window_workgroups(n, p.nch);
    const int ncol = p.ncb * 16;
    const int n16 = threadIdx.x & 15, cl = threadIdx.x >> 4;
    const int col = cb * 16 + n16;
    const int64_t bg = (int64_t)b * p.Hkv + g;
    const float* part = p.part + (bg * p.nch * ncol + col) * 2;
    float m = -INFINITY, l = 0.f;
    for (int c0 = cl; c0 < nchunks; c0 += 64) {            // four loads in flight
        float2 ml[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + 16 * u;
            ml[u] = c < nchunks ? *reinterpret_cast<const float2*>(part + (int64_t)c * ncol * 2) : make_float2(-INFINITY, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) merge_ml(m, l, ml[u].x, ml[u].y);
    }
    __shared__ float sM[16][16], sL[16][16];
    sM[cl][n16] = m; sL[cl][n16] = l;
    __syncthreads();
    if (cl == 0) {
        float M = -INFINITY;
#pragma unroll
        for (int x = 0; x < 16; ++x) M = fmaxf(M, sM[x][n16]);
        double L = 0.0;
#pragma unroll
        for (int x = 0; x < 16; ++x)
            if (sM[x][n16] != -INFINITY) L += (double)fast_exp2((sM[x][n16] - M) * kLog2e) * (double)sL[x][n16];
        float hi = INFINITY, lo = 0.f;                     // a column nobody votes in: e^{s - inf} = 0
        if (M != -INFINITY) {
            const double lse = (double)M + log(L);
            hi = (float)lse; lo = (float)(lse - (double)hi);
        }
        *reinterpret_cast<float2*>(p.lse + (bg * ncol + col) * 2) = make_float2(hi, lo);
    }
}

// Pass 2.
__global__ __launch_bounds__(kWinWaves * 64)
void window_vote_kernel(const WindowParams p) {
    constexpr int NW = kWinWaves;
    const int ncb = p.ncb, NCOL = ncb * 16;
    const int c = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    if (p.pred != nullptr && p.pred[b] != p.pred_val) return;
    const int n = min(max(min(p.seq_lens[b], p.cap), 0), p.max_rows);
    if (n == 0 || c >= window_workgroups(n, p.nch)) return;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n16 = lane & 15, c4 = lane >> 4;
    uint16_t* sQ = reinterpret_cast<uint16_t*>(window_lds);
    float2* sLse = reinterpret_cast<float2*>(window_lds + (size_t)NCOL * kQStride * 2);   // [NCOL]
    const int64_t bg = (int64_t)b * p.Hkv + g;
    stage_queries(p, b, g, n, NCOL, sQ);
    for (int col = tid; col < NCOL; col += NW * 64) sLse[col] = *reinterpret_cast<const float2*>(p.lse + (bg * NCOL + col) * 2);
    __syncthreads();

    const uint16_t* kb = p.k + (int64_t)b * p.s_b + (int64_t)g * p.s_h + c4 * 8;
    const int step = p.nch * NW * kWinRows;
    const int gp = 1 << p.gp_shift;
    float* vrow = p.votes + ((int64_t)b * p.Hq + (int64_t)g * p.G + (n16 < p.G ? n16 : 0)) * p.v_stride;

    u32x4 kA[2][4], kB[2][4];
    auto tile = [&](const u32x4 (&k)[2][4], int r) {
        float v[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll 1
        for (int cb = 0; cb < ncb; ++cb) {
            float s[2][4];
            const int limit = column_limit(p, cb * 16 + n16, n);
            tile_scores(k, sQ, cb, n16, c4, r, limit, p.scale, s);
            const float2 lse = sLse[cb * 16 + n16];
#pragma unroll
            for (int e = 0; e < 8; ++e)                    // s = -inf (masked) gives 2^-inf = 0
                v[e >> 2][e & 3] += fast_exp2(((s[e >> 2][e & 3] - lse.x) - lse.y) * kLog2e);
        }
        // lanes n16, n16 + Gp, n16 + 2 Gp ... hold the same head for different queries
        for (int x = gp; x < 16; x <<= 1) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e >> 2][e & 3] += __shfl_xor(v[e >> 2][e & 3], x);
        }
        if (n16 < p.G) {
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int first = r + t * 16 + 4 * c4;
                if (p.v_vec && first + 4 <= n) {
                    *reinterpret_cast<float4*>(vrow + first) = make_float4(v[t][0], v[t][1], v[t][2], v[t][3]);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (first + i < n) vrow[first + i] = v[t][i];
                }
            }
        }
    };
    int r = (c * NW + w) * kWinRows;
    if (r < n) load_k_tile(kA, kb, r, n16, n);
    if (r + step < n) load_k_tile(kB, kb, r + step, n16, n);
    while (r < n) {
        tile(kA, r);
        if (r + 2 * step < n) load_k_tile(kA, kb, r + 2 * step, n16, n);
        r += step;
        if (r >= n) break;
        tile(kB, r);
        if (r + 2 * step < n) load_k_tile(kB, kb, r + 2 * step, n16, n);
        r += step;
    }
}

static int launch_window(const WindowParams& p, int batch, hipStream_t st) {
    const size_t ncol = (size_t)p.ncb * 16, nt = kWinWaves * 64;
    const size_t lds1 = ncol * kQStride * 2 + p.ncb * nt * sizeof(float2) + 2 * kWinWaves * ncol * sizeof(float);
    const size_t lds2 = ncol * kQStride * 2 + ncol * sizeof(float2);
    static size_t lds_allowed = 48 * 1024;       // grows monotonically; lds1 > lds2
    if (lds1 > lds_allowed) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&window_lse_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(&window_vote_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1) != hipSuccess) {
            (void)hipGetLastError();
            return RK_ERR_UNSUPPORTED;
        }
        lds_allowed = lds1;
    }
    dim3 grid(p.nch, p.Hkv, batch);
    hipLaunchKernelGGL(window_lse_kernel, grid, dim3(kWinWaves * 64), lds1, st, p);
    int rc = launch_status();
    if (rc != RK_OK) return rc;
    hipLaunchKernelGGL(window_lse_merge_kernel, dim3(p.ncb, p.Hkv, batch), dim3(256), 0, st, p);
    if ((rc = launch_status()) != RK_OK) return rc;
    hipLaunchKernelGGL(window_vote_kernel, grid, dim3(kWinWaves * 64), lds2, st, p);
    return launch_status();
}

}  // namespace rk

using namespace rk;

extern "C" int rk_window_select(const rk_geom* geom, const void* q_win, int32_t window, rk_kv full,
                                const int32_t* seq_lens, int32_t max_len,
                                float* votes, int64_t v_stride,
                                int32_t k, int32_t pool_w, int32_t agg,
                                int32_t* idx, float* sel_scores,
                                const int32_t* pred, int32_t pred_val,
                                void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!q_win || !seq_lens || !idx || max_len <= 0 || k <= 0 || window <= 0) return RK_ERR_INVALID_ARG;
    if (window > RK_MAX_WINDOW) return RK_ERR_UNSUPPORTED;
    if (!aligned16(q_win)) return RK_ERR_INVALID_ARG;
    if ((rc = check_kv(full, false)) != RK_OK) return rc;
    if (votes && (v_stride < max_len || ((uintptr_t)votes & 3u))) return RK_ERR_INVALID_ARG;
    if ((rc = check_select_args(k, pool_w, agg, max_len)) != RK_OK) return rc;
    Workspace ws;
    if ((rc = check_workspace(geom, max_len, k, workspace, workspace_bytes, &ws)) != RK_OK) return rc;
    hipStream_t st = (hipStream_t)stream;

    const int G = geom->n_q_heads / geom->n_kv_heads;
    int gp_shift = 0;
    while ((1 << gp_shift) < G) ++gp_shift;
    const int blocks = ((window << gp_shift) + 15) / 16;           // blocks of 16 columns in use
    const int ncb = blocks;
    // the per-workgroup (max, sum) pairs borrow the partial-output area, the column lse the area of
    // the decode kernels' (max, sum) pairs: both are free between calls
    if ((size_t)ncb * 16 * 2 > (size_t)G * kD || (size_t)ncb * 16 > (size_t)kMaxChunks * G) return RK_ERR_UNSUPPORTED;

    WindowParams p{};
    p.q = (const uint16_t*)q_win;
    p.k = (const uint16_t*)full.k; p.s_b = full.stride_b; p.s_h = full.stride_h; p.cap = (int32_t)full.capacity;
    p.seq_lens = seq_lens; p.max_rows = max_len;
    p.W = window; p.G = G; p.gp_shift = gp_shift;
    p.nch = split_workgroups(max_len, (int64_t)geom->batch * geom->n_kv_heads, ws.max_chunks);
    p.Hq = geom->n_q_heads; p.Hkv = geom->n_kv_heads;
    p.scale = geom->scale;
    p.part = ws.part_o; p.lse = ws.part_ml;
    if (votes) { p.votes = votes; p.v_stride = v_stride; }
    else       { p.votes = ws.scores; p.v_stride = pooled_row_stride(max_len); }
    p.v_vec = ((p.v_stride % 4 == 0) && aligned16(p.votes)) ? 1 : 0;
    p.pred = pred; p.pred_val = pred_val;
    p.ncb = ncb;
    rc = launch_window(p, geom->batch, st);
    if (rc != RK_OK) return rc;
    if ((rc = pool_stage(geom, p.votes, p.v_stride, seq_lens, max_len, pool_w, agg, pred, pred_val, ws, st)) != RK_OK) return rc;
    return select_stage(geom, seq_lens, max_len, k, idx, sel_scores, pred, pred_val, ws, st);
}
