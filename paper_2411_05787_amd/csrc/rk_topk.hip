// rk_topk_select for gfx950: group max + max-pool, then an exact, tie-correct top-K.
//
// Kernel 1 (whole chip): P[j] = max over the G heads of the group and over the pooling window
//   of the attention weights, staged through LDS so that every weight is read once.
// Kernel 2 (one workgroup per (sequence, KV head)): radix select on the order-preserving
//   32-bit image of P (three histogram passes: 11 + 11 + 10 bits) finds the K-th largest value
//   T exactly; every position with P > T is taken, positions with P == T are taken in
//   ascending position until K are reached; the winners are then sorted in LDS (bitonic) on
//   the 64-bit key (P image, ~position), which is the required order: score descending, equal
//   scores by ascending position.  Integer comparisons only: the result is exact.
#include "rk_internal.h"
#include "rk_device.h"

namespace rk {

constexpr int kPoolTile = 1024;
constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

__global__ __launch_bounds__(256)
void pool_scores_kernel(const float* __restrict__ weights, int64_t w_stride, const int32_t* seq_lens,
                        int32_t max_len, int32_t Hq, int32_t Hkv, int32_t G, int32_t half,
                        float* __restrict__ pooled, int64_t pooled_stride,
                        const int32_t* pred, int32_t pred_val) {
    const int g = blockIdx.y, b = blockIdx.z;
    if (pred != nullptr && pred[b] != pred_val) return;
    const int len = min(seq_lens[b], max_len);
    const int j0 = blockIdx.x * kPoolTile;
    if (j0 >= len) return;
    __shared__ float sA[kPoolTile + RK_MAX_POOL_W - 1];
    const float* wg = weights + ((int64_t)b * Hq + (int64_t)g * G) * w_stride;
    const int span = kPoolTile + 2 * half;
    for (int i = threadIdx.x; i < span; i += 256) {
        const int j = j0 - half + i;
        float a = -INFINITY;                     // outside [0, len): never wins a max
        if (j >= 0 && j < len) {
            a = wg[j];
            for (int gi = 1; gi < G; ++gi) a = fmaxf(a, wg[(int64_t)gi * w_stride + j]);
        }
        sA[i] = a;
    }
    __syncthreads();
    float* out = pooled + ((int64_t)b * Hkv + g) * pooled_stride;
    for (int i = threadIdx.x; i < kPoolTile; i += 256) {
        const int j = j0 + i;
        if (j < len) {
            float m = sA[i];
            for (int d = 1; d <= 2 * half; ++d) m = fmaxf(m, sA[i + d]);
            out[j] = m + 0.0f;                   // -0 becomes +0: one bit pattern per value
        }
    }
}

// Order-preserving map float -> uint32 (larger float <=> larger key) and its inverse.
__device__ __forceinline__ uint32_t key_of(float x) {
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float value_of(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Inclusive prefix sum over the kSelThreads threads of the workgroup, in thread order.
// `scratch` holds kSelWaves + 1 words.  Returns the inclusive sum; *total gets the block sum.
__device__ __forceinline__ uint32_t block_inclusive_scan(uint32_t v, uint32_t* scratch, uint32_t* total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t x = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t y = __shfl_up(x, d);
        if (lane >= d) x += y;
    }
    __syncthreads();                              // scratch may still be read from a previous scan
    if (lane == 63) scratch[w] = x;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kSelWaves; ++i) {
        const uint32_t s = scratch[i];
        if (i < w) base += s;
        tot += s;
    }
    *total = tot;
    return x + base;
}

// One histogram pass of the radix select.  On entry the keys still in play are those with
// (key & mask) == prefix and the kk-th largest of them is wanted.  Bins are `bits` wide at
// `shift`.  Returns through LDS (sOut[0] = bin holding the kk-th largest, sOut[1] = number of
// candidates in higher bins).
template <int BITS>
__device__ void radix_pass(const float* __restrict__ P, int n, uint32_t prefix, uint32_t mask, int shift,
                           uint32_t kk, uint32_t* sHist, uint32_t* sScan, uint32_t* sOut) {
    constexpr int NB = 1 << BITS;
    constexpr int BPT = NB / kSelThreads;          // bins per thread: 2 (11 bits) or 1 (10 bits)
    static_assert(BPT >= 1, "at least one bin per thread");
    const int tid = threadIdx.x;
    for (int i = tid; i < NB; i += kSelThreads) sHist[i] = 0;
    __syncthreads();
    for (int j = tid; j < n; j += kSelThreads) {
        const uint32_t key = key_of(P[j]);
        if ((key & mask) == prefix) atomicAdd(&sHist[(key >> shift) & (NB - 1)], 1u);
    }
    __syncthreads();
    // thread t owns bins [BPT*t, BPT*t + BPT); scan from the top: reverse the thread order
    const int rt = kSelThreads - 1 - tid;
    uint32_t local = 0;
#pragma unroll
    for (int i = 0; i < BPT; ++i) local += sHist[rt * BPT + i];
    uint32_t total;
    const uint32_t incl = block_inclusive_scan(local, sScan, &total);   // bins >= BPT*rt
    uint32_t above = incl - local;                                       // bins >= BPT*(rt+1)
    if (above < kk && kk <= incl) {
#pragma unroll
        for (int i = BPT - 1; i >= 0; --i) {
            const uint32_t h = sHist[rt * BPT + i];
            if (above + h >= kk) { sOut[0] = (uint32_t)(rt * BPT + i); sOut[1] = above; break; }
            above += h;
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(kSelThreads)
void select_kernel(const float* __restrict__ pooled, int64_t pooled_stride, const int32_t* seq_lens,
                   int32_t max_len, int32_t k, int32_t kpad_max, int32_t* __restrict__ idx,
                   float* __restrict__ sel_scores, const int32_t* pred, int32_t pred_val) {
    const int g = blockIdx.x, b = blockIdx.y, Hkv = gridDim.x;
    if (pred != nullptr && pred[b] != pred_val) return;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint64_t* sKeys = reinterpret_cast<uint64_t*>(smem);                   // [kpad_max]
    uint32_t* sHist = reinterpret_cast<uint32_t*>(sKeys + kpad_max);       // [2048]
    uint32_t* sScan = sHist + 2048;                                        // [kSelWaves]
    uint32_t* sOut = sScan + kSelWaves;                                    // [2]
    uint32_t* sCount = sOut + 2;                                           // [1]

    const int tid = threadIdx.x;
    const int n = min(seq_lens[b], max_len);
    const int kprime = min(k, max(n, 0));
    const int64_t ob = ((int64_t)b * Hkv + g) * k;
    if (kprime <= 0) {
        for (int i = tid; i < k; i += kSelThreads) { idx[ob + i] = -1; if (sel_scores) sel_scores[ob + i] = 0.f; }
        return;
    }
    const float* P = pooled + ((int64_t)b * Hkv + g) * pooled_stride;

    // ---- exact K-th largest key T ----
    uint32_t prefix = 0, mask = 0, kk = (uint32_t)kprime;
    radix_pass<11>(P, n, prefix, mask, 21, kk, sHist, sScan, sOut);
    prefix |= sOut[0] << 21; mask |= 0x7FFu << 21; kk -= sOut[1];
    __syncthreads();
    radix_pass<11>(P, n, prefix, mask, 10, kk, sHist, sScan, sOut);
    prefix |= sOut[0] << 10; mask |= 0x7FFu << 10; kk -= sOut[1];
    __syncthreads();
    radix_pass<10>(P, n, prefix, mask, 0, kk, sHist, sScan, sOut);
    const uint32_t T = prefix | sOut[0];
    const uint32_t need_eq = kk - sOut[1];          // >= 1 positions with key == T are taken
    const uint32_t n_gt = (uint32_t)kprime - need_eq;
    if (tid == 0) *sCount = 0;
    __syncthreads();

    // ---- collect: every key > T, and the first need_eq positions with key == T ----
    uint32_t base_eq = 0;
    for (int tile0 = 0; tile0 < n; tile0 += kSelThreads) {
        const int j = tile0 + tid;
        const bool in = j < n;
        const uint32_t key = in ? key_of(P[j]) : 0u;
        const uint64_t item = ((uint64_t)key << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)j);
        if (in && key > T) sKeys[atomicAdd(sCount, 1u)] = item;
        const bool eq = in && key == T;
        if (base_eq < need_eq) {                    // uniform over the workgroup
            if (__syncthreads_or(eq ? 1 : 0)) {
                uint32_t total;
                const uint32_t incl = block_inclusive_scan(eq ? 1u : 0u, sScan, &total);
                const uint32_t rank = base_eq + incl - 1u;
                if (eq && rank < need_eq) sKeys[n_gt + rank] = item;
                base_eq += total;
            }
        }
    }
    int kpad = 1;
    while (kpad < kprime) kpad <<= 1;
    for (int i = kprime + tid; i < kpad; i += kSelThreads) sKeys[i] = 0;   // sorts behind every real item
    __syncthreads();

    // ---- bitonic sort, descending ----
    for (int size = 2; size <= kpad; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int i = tid; i < (kpad >> 1); i += kSelThreads) {
                const int lo = ((i & ~(stride - 1)) << 1) | (i & (stride - 1));
                const int hi = lo + stride;
                const bool desc = (lo & size) == 0;
                const uint64_t a = sKeys[lo], c = sKeys[hi];
                if ((a < c) == desc) { sKeys[lo] = c; sKeys[hi] = a; }
            }
            __syncthreads();
        }
    }
    for (int i = tid; i < k; i += kSelThreads) {
        if (i < kprime) {
            const uint64_t item = sKeys[i];
            idx[ob + i] = (int32_t)(0xFFFFFFFFu - (uint32_t)(item & 0xFFFFFFFFu));
            if (sel_scores) sel_scores[ob + i] = value_of((uint32_t)(item >> 32));
        } else {
            idx[ob + i] = -1;
            if (sel_scores) sel_scores[ob + i] = 0.f;
        }
    }
}

}  // namespace rk

using namespace rk;

extern "C" int rk_topk_select(const rk_geom* geom, const float* weights, int64_t w_stride,
                              const int32_t* seq_lens, int32_t max_len,
                              int32_t k, int32_t pool_w, int32_t agg,
                              int32_t* idx, float* sel_scores,
                              const int32_t* pred, int32_t pred_val,
                              void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!weights || !seq_lens || !idx || max_len <= 0 || k <= 0 || w_stride < max_len) return RK_ERR_INVALID_ARG;
    if (pool_w < 1 || (pool_w & 1) == 0) return RK_ERR_INVALID_ARG;
    if (pool_w > RK_MAX_POOL_W || k > RK_MAX_K || agg != RK_AGG_MAX) return RK_ERR_UNSUPPORTED;
    Workspace ws;
    if ((rc = check_workspace(geom, max_len, k, workspace, workspace_bytes, &ws)) != RK_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int G = geom->n_q_heads / geom->n_kv_heads;

    dim3 pgrid((max_len + kPoolTile - 1) / kPoolTile, geom->n_kv_heads, geom->batch);
    hipLaunchKernelGGL(pool_scores_kernel, pgrid, dim3(256), 0, st, weights, w_stride, seq_lens, max_len,
                       geom->n_q_heads, geom->n_kv_heads, G, (pool_w - 1) / 2, ws.pooled, (int64_t)max_len,
                       pred, pred_val);
    if ((rc = launch_status()) != RK_OK) return rc;

    int kpad = 1;
    while (kpad < k) kpad <<= 1;
    const size_t lds = (size_t)kpad * sizeof(uint64_t) + (2048 + kSelWaves + 2 + 1) * sizeof(uint32_t);
    static size_t lds_allowed = 48 * 1024;       // grows monotonically; set before the first large launch
    if (lds > lds_allowed) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&select_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return RK_ERR_UNSUPPORTED;
        }
        lds_allowed = lds;
    }
    dim3 sgrid(geom->n_kv_heads, geom->batch);
    hipLaunchKernelGGL(select_kernel, sgrid, dim3(kSelThreads), lds, st, ws.pooled, (int64_t)max_len, seq_lens,
                       max_len, k, kpad, idx, sel_scores, pred, pred_val);
    return launch_status();
}
