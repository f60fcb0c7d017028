// rk_query_sim for gfx950: cosine similarity between the head-averaged query of this step and
// the one stored at the most recent full step.  One workgroup of 128 threads (one per dim) per
// sequence; the whole call moves ~9 KB, so it is launch-latency bound by nature.
#include "rk_internal.h"
#include "rk_device.h"

namespace rk {

__global__ __launch_bounds__(128)
void query_sim_kernel(const uint16_t* __restrict__ q, float* __restrict__ q_ref, int32_t Hq, float threshold,
                      int32_t force_full, float* __restrict__ sim, int32_t* __restrict__ need_full) {
    const int b = blockIdx.x, d = threadIdx.x;
    __shared__ float red[2];
    const uint16_t* qb = q + (int64_t)b * Hq * kD + d;
    const float ref = q_ref[(int64_t)b * kD + d];
    // the heads are added in order; their loads are requested sixteen at a time (one after the
    // other, each waiting for the one before, the kernel took 28 memory round trips at 28 heads)
    float acc = 0.f;
    for (int h0 = 0; h0 < Hq; h0 += 16) {
        uint16_t v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = qb[(int64_t)min(h0 + i, Hq - 1) * kD];
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (h0 + i < Hq) acc += __uint_as_float((uint32_t)v[i] << 16);
    }
    const float qbar = acc / (float)Hq;
    const float dot = block_sum<2>(qbar * ref, red);
    const float n1 = block_sum<2>(qbar * qbar, red);
    const float n2 = block_sum<2>(ref * ref, red);
    const float s = dot / (fmaxf(sqrtf(n1), 1e-8f) * fmaxf(sqrtf(n2), 1e-8f));
    const bool need = !(s > threshold) || force_full != 0;
    if (need) q_ref[(int64_t)b * kD + d] = qbar;
    if (d == 0) { sim[b] = s; need_full[b] = need ? 1 : 0; }
}

}  // namespace rk

using namespace rk;

extern "C" int rk_query_sim(const rk_geom* geom, const void* q, float* q_ref, float threshold,
                            int32_t force_full, float* sim, int32_t* need_full, void* stream) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!q || !q_ref || !sim || !need_full) return RK_ERR_INVALID_ARG;
    hipLaunchKernelGGL(query_sim_kernel, dim3(geom->batch), dim3(128), 0, (hipStream_t)stream,
                       (const uint16_t*)q, q_ref, geom->n_q_heads, threshold, force_full, sim, need_full);
    return launch_status();
}
