// Entry points that launch no compute: version, status strings, workspace sizing and set-up.
#include "rk_internal.h"

using namespace rk;

extern "C" int rk_version(void) { return 100; }   // 0.1.0

extern "C" const char* rk_status_string(int status) {
    switch (status) {
        case RK_OK: return "ok";
        case RK_ERR_INVALID_ARG: return "invalid argument";
        case RK_ERR_UNSUPPORTED: return "unsupported configuration";
        case RK_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case RK_ERR_HIP: return "HIP runtime error";
        case RK_ERR_STATIC_SCRATCH: return "sizes beyond the library's built-in scratch array";
        default: return "unknown status";
    }
}

extern "C" size_t rk_workspace_bytes(const rk_geom* geom, int32_t max_len, int32_t max_k) {
    if (check_geom(geom) != RK_OK || max_len <= 0 || max_k < 0) return 0;
    return carve(geom, max_len, max_k, nullptr).total;
}

namespace rk {
// A fill kernel instead of hipMemsetAsync, so that the call can sit inside a captured graph.
__global__ __launch_bounds__(256) void zero_fill_kernel(uint4* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = make_uint4(0, 0, 0, 0);
}
__global__ __launch_bounds__(256) void calibration_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// Reads n 16-byte words and keeps nothing: what a kernel that only streams from memory reaches on
// this chip (streaming loads, eight in flight per lane, as the full-cache attention kernel issues them).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void calibration_read_kernel(const u32x4_t* __restrict__ src, size_t n, uint32_t* sink) {
    constexpr int UN = 8;
    uint32_t acc = 0;
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + (UN - 1) * stride < n; i += UN * stride) {
        u32x4_t v[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < UN; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < n; i += stride) { const u32x4_t v = __builtin_nontemporal_load(src + i); acc ^= v.x ^ v.y ^ v.z ^ v.w; }
    if (acc == 0x9E3779B9u) sink[0] = acc;       // (keeps the loads; one lane in 2^32 writes)
}

__global__ void mark_refresh_kernel(const int32_t* seq_lens, int32_t* tail_start, int32_t batch,
                                    const int32_t* pred, int32_t pred_val) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < batch && (pred == nullptr || pred[b] == pred_val)) tail_start[b] = seq_lens[b];
}
}  // namespace rk

extern "C" int rk_calibration_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src || bytes == 0 || bytes % 16 != 0 || !aligned16(dst) || !aligned16(src)) return RK_ERR_INVALID_ARG;
    const size_t n = bytes / 16;
    const unsigned grid = (unsigned)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    hipLaunchKernelGGL(calibration_copy_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (uint4*)dst, (const uint4*)src, n);
    return launch_status();
}

extern "C" int rk_calibration_read(const void* src, size_t bytes, uint32_t* sink, void* stream) {
    if (!src || !sink || bytes == 0 || bytes % 16 != 0 || !aligned16(src)) return RK_ERR_INVALID_ARG;
    const size_t n = bytes / 16;
    const unsigned grid = (unsigned)((n + 255) / 256 < 8192 ? (n + 255) / 256 : 8192);
    hipLaunchKernelGGL(calibration_read_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const u32x4_t*)src, n, sink);
    return launch_status();
}

extern "C" int rk_mark_refresh(const rk_geom* geom, const int32_t* seq_lens, int32_t* tail_start,
                               const int32_t* pred, int32_t pred_val, void* stream) {
    if (check_geom(geom) != RK_OK || !seq_lens || !tail_start) return RK_ERR_INVALID_ARG;
    hipLaunchKernelGGL(mark_refresh_kernel, dim3((geom->batch + 63) / 64), dim3(64), 0, (hipStream_t)stream,
                       seq_lens, tail_start, geom->batch, pred, pred_val);
    return launch_status();
}

extern "C" int rk_workspace_init(const rk_geom* geom, void* workspace, size_t workspace_bytes, void* stream) {
    if (check_geom(geom) != RK_OK) return RK_ERR_INVALID_ARG;
    if (!workspace || ((uintptr_t)workspace & 255u) != 0) return RK_ERR_WORKSPACE;
    // counters, call numbers, histograms and the tags of the partial results must start at zero; the
    // whole workspace is cleared, so that nothing depends on what the memory held before
    if (workspace_bytes < zero_kept_bytes(geom)) return RK_ERR_WORKSPACE;
    const size_t n = workspace_bytes / 16;
    const unsigned grid = (unsigned)((n + 255) / 256 < 2048 ? (n + 255) / 256 : 2048);
    hipLaunchKernelGGL(zero_fill_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (uint4*)workspace, n);
    return launch_status();
}
