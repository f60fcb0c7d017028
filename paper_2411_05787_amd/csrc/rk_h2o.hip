// The H2O comparison policy on the library's attention step: rk_h2o_append, rk_h2o_update,
// rk_h2o_step (Section 3 "Comparison systems"; Appendix A.1 "Baseline Settings").
//
// A step = append the new token's rows to the policy's cache, attend over the whole cache with
// the scores returned (rk_full_attn's kernels on a cache of at most budget + 1 rows), then one
// small kernel per (sequence, KV head): add the group-aggregated scores to the running totals
// and, when the cache is over its budget, drop the token with the lowest total among those that
// are not recent.  Slots are not kept in token order (attention does not care): the newest
// token, always in the last slot, moves into the slot of the dropped one, so the cache stays
// dense without shifting rows.
#include "rk_internal.h"
#include "rk_device.h"

namespace rk {

constexpr int kH2oThreads = 1024;

__global__ __launch_bounds__(64)
void h2o_append_kernel(rk_h2o_state st, const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new,
                       const int32_t* __restrict__ seq_lens, int32_t Hkv, int64_t meta_stride) {
    const int g = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    const int cap = (int)st.cache.capacity;
    const int slot = min(max(st.n_rows[b], 0), cap - 1);
    const int64_t bg = (int64_t)b * Hkv + g;
    const uint32_t* ks = reinterpret_cast<const uint32_t*>(k_new + bg * kD);
    const uint32_t* vs = reinterpret_cast<const uint32_t*>(v_new + bg * kD);
    uint16_t* kc = (uint16_t*)st.cache.k + (int64_t)b * st.cache.stride_b + (int64_t)g * st.cache.stride_h + (int64_t)slot * kD;
    uint16_t* vc = (uint16_t*)st.cache.v + (int64_t)b * st.cache.stride_b + (int64_t)g * st.cache.stride_h + (int64_t)slot * kD;
    reinterpret_cast<uint32_t*>(kc)[lane] = ks[lane];
    reinterpret_cast<uint32_t*>(vc)[lane] = vs[lane];
    if (lane == 0) {
        st.total[bg * meta_stride + slot] = 0.f;
        st.pos[bg * meta_stride + slot] = seq_lens[b] - 1;
        st.n_attend[b] = slot + 1;                 // every head of the sequence writes the same value
    }
}

// 64-bit minimum over the workgroup; `red` holds kH2oThreads / 64 words.  Every thread gets it.
__device__ __forceinline__ uint64_t block_min_u64(uint64_t v, uint64_t* red) {
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        const uint64_t o = __shfl_xor(v, m);
        v = o < v ? o : v;
    }
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    uint64_t r = red[0];
    for (int i = 1; i < kH2oThreads / 64; ++i) r = red[i] < r ? red[i] : r;
    return r;
}

__global__ __launch_bounds__(kH2oThreads)
void h2o_update_kernel(rk_h2o_state st, const float* __restrict__ weights, int64_t w_stride, int32_t max_rows,
                       int32_t Hq, int32_t Hkv, int32_t G, int32_t budget, int32_t recent, int32_t agg,
                       int32_t* __restrict__ dropped, int64_t meta_stride) {
    const int g = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int cap = (int)st.cache.capacity;
    const int n = min(min(max(st.n_attend[b], 0), cap), max_rows);
    const int64_t bg = (int64_t)b * Hkv + g;
    float* total = st.total + bg * meta_stride;
    int32_t* pos = st.pos + bg * meta_stride;
    const float* wg = weights + ((int64_t)b * Hq + (int64_t)g * G) * w_stride;
    __shared__ uint64_t red[kH2oThreads / 64];
    __shared__ int sVictim;
    const bool over = n > budget;
    const int newest = n > 0 ? pos[n - 1] : 0;
    uint64_t best = ~0ull;
    for (int j = tid; j < n; j += kH2oThreads) {
        float a = -INFINITY;
        for (int gi = 0; gi < G; ++gi) a = aggregate(a, wg[(int64_t)gi * w_stride + j], gi, agg);
        if (agg == RK_AGG_MEAN) a = __fdiv_rn(a, (float)G);
        const float t = __fadd_rn(total[j], a);
        total[j] = t;
        const int pj = pos[j];
        if (over && pj <= newest - recent) {       // lowest total first, the older token on equal totals
            const uint64_t key = ((uint64_t)key_of(t) << 32) | (uint32_t)pj;
            best = key < best ? key : best;
        }
    }
    if (tid == 0) sVictim = -1;
    best = block_min_u64(best, red);               // has a barrier after the write of sVictim
    int32_t gone = -1;
    if (over && best != ~0ull) {
        gone = (int32_t)(uint32_t)best;
        for (int j = tid; j < n; j += kH2oThreads)
            if (pos[j] == gone) sVictim = j;       // positions are unique within a cache
        __syncthreads();
        const int v = sVictim, last = n - 1;
        if (v >= 0 && v != last) {
            uint16_t* kc = (uint16_t*)st.cache.k + (int64_t)b * st.cache.stride_b + (int64_t)g * st.cache.stride_h;
            uint16_t* vc = (uint16_t*)st.cache.v + (int64_t)b * st.cache.stride_b + (int64_t)g * st.cache.stride_h;
            if (tid < 64)        reinterpret_cast<uint32_t*>(kc + (int64_t)v * kD)[tid] = reinterpret_cast<const uint32_t*>(kc + (int64_t)last * kD)[tid];
            else if (tid < 128)  reinterpret_cast<uint32_t*>(vc + (int64_t)v * kD)[tid - 64] = reinterpret_cast<const uint32_t*>(vc + (int64_t)last * kD)[tid - 64];
            else if (tid == 128) { total[v] = total[last]; pos[v] = pos[last]; }
        }
    }
    if (tid == 0) {
        if (dropped) dropped[bg] = gone;
        st.n_rows[b] = gone >= 0 ? n - 1 : n;      // every head of the sequence writes the same value
    }
}

static int check_h2o(const rk_geom* geom, const rk_h2o_state& st, int32_t budget, int32_t recent) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if ((rc = check_kv(st.cache)) != RK_OK) return rc;
    if (!st.total || !st.pos || !st.n_rows || !st.n_attend) return RK_ERR_INVALID_ARG;
    if (budget <= 0 || recent < 0 || recent >= budget) return RK_ERR_INVALID_ARG;
    if (st.cache.capacity < (int64_t)budget + 1) return RK_ERR_INVALID_ARG;
    return RK_OK;
}

static int append_stage(const rk_geom* geom, const rk_h2o_state& st, const void* k_new, const void* v_new,
                        const int32_t* seq_lens, hipStream_t s) {
    hipLaunchKernelGGL(h2o_append_kernel, dim3(geom->n_kv_heads, geom->batch), dim3(64), 0, s, st,
                       (const uint16_t*)k_new, (const uint16_t*)v_new, seq_lens, geom->n_kv_heads, st.cache.capacity);
    return launch_status();
}

static int update_stage(const rk_geom* geom, const rk_h2o_state& st, const float* weights, int64_t w_stride,
                        int32_t max_rows, int32_t budget, int32_t recent, int32_t agg, int32_t* dropped, hipStream_t s) {
    hipLaunchKernelGGL(h2o_update_kernel, dim3(geom->n_kv_heads, geom->batch), dim3(kH2oThreads), 0, s, st,
                       weights, w_stride, max_rows, geom->n_q_heads, geom->n_kv_heads, geom->n_q_heads / geom->n_kv_heads,
                       budget, recent, agg, dropped, st.cache.capacity);
    return launch_status();
}

}  // namespace rk

using namespace rk;

extern "C" int rk_h2o_append(const rk_geom* geom, rk_h2o_state state, const void* k_new, const void* v_new,
                             const int32_t* seq_lens, int32_t budget, void* stream) {
    int rc = check_h2o(geom, state, budget, 0);
    if (rc != RK_OK) return rc;
    if (!k_new || !v_new || !seq_lens || ((uintptr_t)k_new & 3u) || ((uintptr_t)v_new & 3u)) return RK_ERR_INVALID_ARG;
    return append_stage(geom, state, k_new, v_new, seq_lens, (hipStream_t)stream);
}

extern "C" int rk_h2o_update(const rk_geom* geom, rk_h2o_state state, const float* weights, int64_t w_stride,
                             int32_t budget, int32_t recent, int32_t agg, int32_t* dropped, void* stream) {
    int rc = check_h2o(geom, state, budget, recent);
    if (rc != RK_OK) return rc;
    if (!weights || w_stride < (int64_t)budget + 1 || ((uintptr_t)weights & 3u)) return RK_ERR_INVALID_ARG;
    if (agg < RK_AGG_MAX || agg > RK_AGG_FIRST) return RK_ERR_UNSUPPORTED;
    return update_stage(geom, state, weights, w_stride, budget + 1, budget, recent, agg, dropped, (hipStream_t)stream);
}

extern "C" int rk_h2o_step(const rk_geom* geom, rk_h2o_state state, const void* q,
                           const void* k_new, const void* v_new, const int32_t* seq_lens,
                           int32_t budget, int32_t recent, int32_t agg,
                           void* out, int32_t* dropped,
                           void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_h2o(geom, state, budget, recent);
    if (rc != RK_OK) return rc;
    if (!q || !out || !k_new || !v_new || !seq_lens) return RK_ERR_INVALID_ARG;
    if (!aligned16(q) || ((uintptr_t)out & 1u) || ((uintptr_t)k_new & 3u) || ((uintptr_t)v_new & 3u)) return RK_ERR_INVALID_ARG;
    if (agg < RK_AGG_MAX || agg > RK_AGG_FIRST) return RK_ERR_UNSUPPORTED;
    const int32_t max_rows = budget + 1;
    Workspace ws;
    if ((rc = check_workspace(geom, max_rows, 0, workspace, workspace_bytes, &ws)) != RK_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    if ((rc = append_stage(geom, state, k_new, v_new, seq_lens, s)) != RK_OK) return rc;
    // the scores of the step go through the workspace's score area (one row per query head)
    const int64_t w_stride = pooled_row_stride(max_rows);
    rc = full_attn_stage(geom, q, state.cache, state.n_attend, max_rows, out, ws.scores, w_stride, nullptr,
                         nullptr, 0, ws, s, false, -1, false, RK_AGG_MAX);
    if (rc != RK_OK) return rc;
    return update_stage(geom, state, ws.scores, w_stride, max_rows, budget, recent, agg, dropped, s);
}
