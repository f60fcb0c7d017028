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

// The gathers of several layers in one launch: grid z = layer * batch + sequence.
struct GatherBatch {
    const uint16_t* fk[kBatchLayers]; const uint16_t* fv[kBatchLayers];
    uint16_t* sk[kBatchLayers]; uint16_t* sv[kBatchLayers];
    const int32_t* idx[kBatchLayers];
    int32_t* tail_start[kBatchLayers]; int32_t* n_refresh[kBatchLayers];
    const int32_t* pred[kBatchLayers];
};

__global__ __launch_bounds__(256)
void gather_rows_batched_kernel(const GatherBatch tab, int32_t batch, int64_t fs_b, int64_t fs_h, int64_t ss_b, int64_t ss_h,
                                int32_t k, int32_t Hkv, int32_t full_cap, const int32_t* __restrict__ seq_lens,
                                int32_t pred_val) {
    const int layer = blockIdx.z / batch, b = blockIdx.z - layer * batch, g = blockIdx.y;
    if (tab.pred[layer] != nullptr && tab.pred[layer][b] != pred_val) return;
    if (blockIdx.x == 0 && g == 0 && threadIdx.x == 0) {
        if (tab.tail_start[layer] != nullptr) tab.tail_start[layer][b] = seq_lens[b];
        if (tab.n_refresh[layer] != nullptr) tab.n_refresh[layer][b] += 1;
    }
    const int i = blockIdx.x * kGatherRows + (threadIdx.x >> 4);
    if (i >= k) return;
    const int j = tab.idx[layer][((int64_t)b * Hkv + g) * k + i];
    if (j < 0 || j >= full_cap) return;
    const int seg = (threadIdx.x & 15) * 8;
    const int64_t src = (int64_t)b * fs_b + (int64_t)g * fs_h + (int64_t)j * kD + seg;
    const int64_t dst = (int64_t)b * ss_b + (int64_t)g * ss_h + (int64_t)i * kD + seg;
    const uint4 kr = *reinterpret_cast<const uint4*>(tab.fk[layer] + src);
    const uint4 vr = *reinterpret_cast<const uint4*>(tab.fv[layer] + src);
    *reinterpret_cast<uint4*>(tab.sk[layer] + dst) = kr;
    *reinterpret_cast<uint4*>(tab.sv[layer] + dst) = vr;
}

}  // namespace rk

namespace rk {
int gather_batched_stage(const rk_geom* geom, int n_layers, const rk_kv* full, const rk_kv* small, int32_t* const* idx,
                         int32_t k, const int32_t* seq_lens, int32_t* const* tail_start, int32_t* const* n_refresh,
                         const int32_t* const* pred, int32_t pred_val, hipStream_t st) {
    if (k <= 0 || !seq_lens) return RK_ERR_INVALID_ARG;
    if ((int64_t)kBatchLayers * geom->batch > 65535) return RK_ERR_UNSUPPORTED;
    for (int l = 0; l < n_layers; ++l) {
        int rc;
        if ((rc = check_kv(full[l])) != RK_OK || (rc = check_kv(small[l])) != RK_OK) return rc;
        if (small[l].capacity < k || !idx[l]) return RK_ERR_INVALID_ARG;
        // one launch takes one set of strides
        if (full[l].stride_b != full[0].stride_b || full[l].stride_h != full[0].stride_h || full[l].capacity != full[0].capacity ||
            small[l].stride_b != small[0].stride_b || small[l].stride_h != small[0].stride_h) return RK_ERR_UNSUPPORTED;
    }
    for (int l0 = 0; l0 < n_layers; l0 += kBatchLayers) {
        const int n = n_layers - l0 < kBatchLayers ? n_layers - l0 : kBatchLayers;
        GatherBatch tab{};
        for (int l = 0; l < n; ++l) {
            tab.fk[l] = (const uint16_t*)full[l0 + l].k; tab.fv[l] = (const uint16_t*)full[l0 + l].v;
            tab.sk[l] = (uint16_t*)small[l0 + l].k; tab.sv[l] = (uint16_t*)small[l0 + l].v;
            tab.idx[l] = idx[l0 + l];
            tab.tail_start[l] = tail_start ? tail_start[l0 + l] : nullptr;
            tab.n_refresh[l] = n_refresh ? n_refresh[l0 + l] : nullptr;
            tab.pred[l] = pred ? pred[l0 + l] : nullptr;
        }
        dim3 grid((k + kGatherRows - 1) / kGatherRows, geom->n_kv_heads, n * geom->batch);
        hipLaunchKernelGGL(gather_rows_batched_kernel, grid, dim3(256), 0, st, tab, (int32_t)geom->batch,
                           full[0].stride_b, full[0].stride_h, small[0].stride_b, small[0].stride_h,
                           k, geom->n_kv_heads, (int32_t)full[0].capacity, seq_lens, pred_val);
        const int rc = launch_status();
        if (rc != RK_OK) return rc;
    }
    return RK_OK;
}

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
