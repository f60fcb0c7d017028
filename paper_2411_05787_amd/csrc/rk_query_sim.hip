// rk_query_sim for gfx950: cosine similarity between the head-averaged query of this step and
// the one stored at the most recent full step.  One wavefront per sequence; the whole call moves
// ~9 KB, so it is launch-latency bound by nature (the partial step of a test step carries the same
// test out itself: rk_partial_attn_triggered).
#include "rk_internal.h"
#include "rk_device.h"

namespace rk {

__global__ __launch_bounds__(64)
void query_sim_kernel(const uint16_t* __restrict__ q, float* q_ref, int32_t Hq, float threshold,
                      int32_t force_full, float* __restrict__ sim, int32_t* __restrict__ need_full) {
    const int b = blockIdx.x, lane = threadIdx.x;
    SimLoads ld;
    similarity_request(q, q_ref, b, Hq, ld);
    float mean[8];
    const float s = similarity_finish(q, b, Hq, ld, mean);
    const bool need = !(s > threshold) || force_full != 0;
    if (need && lane < 16) {
        float4* rp = reinterpret_cast<float4*>(q_ref + (int64_t)b * kD + lane * 8);
        rp[0] = make_float4(mean[0], mean[1], mean[2], mean[3]);
        rp[1] = make_float4(mean[4], mean[5], mean[6], mean[7]);
    }
    if (lane == 0) { sim[b] = s; need_full[b] = need ? 1 : 0; }
}

}  // namespace rk

using namespace rk;

extern "C" int rk_query_sim(const rk_geom* geom, const void* q, float* q_ref, float threshold,
                            int32_t force_full, float* sim, int32_t* need_full, void* stream) {
    int rc = check_geom(geom);
    if (rc != RK_OK) return rc;
    if (!q || !q_ref || !sim || !need_full) return RK_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(q_ref)) return RK_ERR_INVALID_ARG;
    hipLaunchKernelGGL(query_sim_kernel, dim3(geom->batch), dim3(64), 0, (hipStream_t)stream,
                       (const uint16_t*)q, q_ref, geom->n_q_heads, threshold, force_full, sim, need_full);
    return launch_status();
}
