// rk_gather_small_kv for gfx950: copies the selected K and V rows of the full cache into the
// small cache.  A row is 256 bytes: 16 lanes move it with one 16-byte load and store each, so
// a wavefront moves four K rows (or four V rows) per instruction pair.
#include "rk_internal.h"
#include "rk_device.h"

namespace rk {

constexpr int kGatherRows = 16;      // rows per workgroup of 256 threads

__global__ __launch_bounds__(256)
void gather_rows_kernel(const uint16_t* __restrict__ fk, const uint16_t* __restrict__ fv, int64_t fs_b, int64_t fs_h,
                        uint16_t* __restrict__ sk, uint16_t* __restrict__ sv, int64_t ss_b, int64_t ss_h,
                        const int32_t* __restrict__ idx, int32_t k, int32_t Hkv, int32_t full_cap,
                        const int32_t* __restrict__ seq_lens, int32_t* __restrict__ tail_start,
                        int32_t* __restrict__ n_refresh, const int32_t* pred, int32_t pred_val) {
    const int g = blockIdx.y, b = blockIdx.z;
    if (pred != nullptr && pred[b] != pred_val) return;
    if (blockIdx.x == 0 && g == 0 && threadIdx.x == 0) {
        if (tail_start != nullptr) tail_start[b] = seq_lens[b];
        if (n_refresh != nullptr) n_refresh[b] += 1;       // one writer per sequence and launch
    }
    const int i = blockIdx.x * kGatherRows + (threadIdx.x >> 4);
    if (i >= k) return;
    const int j = idx[((int64_t)b * Hkv + g) * k + i];
    if (j < 0 || j >= full_cap) return;
    const int seg = (threadIdx.x & 15) * 8;
    const int64_t src = (int64_t)b * fs_b + (int64_t)g * fs_h + (int64_t)j * kD + seg;
    const int64_t dst = (int64_t)b * ss_b + (int64_t)g * ss_h + (int64_t)i * kD + seg;
    const uint4 kr = *reinterpret_cast<const uint4*>(fk + src);
    const uint4 vr = *reinterpret_cast<const uint4*>(fv + src);
    *reinterpret_cast<uint4*>(sk + dst) = kr;
    *reinterpret_cast<uint4*>(sv + dst) = vr;
}

}  // namespace rk

namespace rk {
int gather_stage(const rk_geom* geom, rk_kv full, const int32_t* idx, int32_t k, rk_kv small,
                 const int32_t* seq_lens, int32_t* tail_start, int32_t* n_refresh,
                 const int32_t* pred, int32_t pred_val, hipStream_t stream) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!idx || k <= 0 || (tail_start && !seq_lens)) return RK_ERR_INVALID_ARG;
    if ((rc = check_kv(full)) != RK_OK) return rc;
    if ((rc = check_kv(small)) != RK_OK) return rc;
    if (small.capacity < k) return RK_ERR_INVALID_ARG;
    dim3 grid((k + kGatherRows - 1) / kGatherRows, geom->n_kv_heads, geom->batch);
    hipLaunchKernelGGL(gather_rows_kernel, grid, dim3(256), 0, stream,
                       (const uint16_t*)full.k, (const uint16_t*)full.v, full.stride_b, full.stride_h,
                       (uint16_t*)small.k, (uint16_t*)small.v, small.stride_b, small.stride_h,
                       idx, k, geom->n_kv_heads, (int32_t)full.capacity, seq_lens, tail_start, n_refresh, pred, pred_val);
    return launch_status();
}
}  // namespace rk

using namespace rk;

extern "C" int rk_gather_small_kv(const rk_geom* geom, rk_kv full, const int32_t* idx, int32_t k,
                                  rk_kv small, const int32_t* seq_lens, int32_t* tail_start,
                                  const int32_t* pred, int32_t pred_val, void* stream) {
    return gather_stage(geom, full, idx, k, small, seq_lens, tail_start, nullptr, pred, pred_val, (hipStream_t)stream);
}
