// Device-side helpers shared by the kernels: bf16 unpacking, wavefront (64 lanes) and
// workgroup reductions, MFMA operand types.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rk {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;

// A dword holds two bf16: element 2i in the low half, 2i+1 in the high half.
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// fp32 -> bf16, round to nearest even; NaN stays a (quiet) NaN.
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// 2^x on the hardware transcendental unit (v_exp_f32); 2^-inf = 0.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Cross-lane reductions without the LDS crossbar.  A shuffle (ds_bpermute) is a round trip through
// the LDS pipeline of its own, and a reduction is a chain of them; the data-parallel-primitive
// operand path of the VALU moves data inside a row of 16 lanes in a few cycles, and gfx950's
// v_permlane16_swap / v_permlane32_swap exchange rows and halves of the wavefront.  It matters
// where nothing hides the chain: the tile of a partial step, a merge that one workgroup runs alone
// (8.81 -> 8.58 us per partial step at K = 2048).  All 64 lanes must be active at every call.
template <int CTRL>
__device__ __forceinline__ int dpp_move(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false); }
// lane ^ 1 and lane ^ 2 inside every quad; the row of 16 rotated by 4 and by 8
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppRor4 = 0x124, kDppRor8 = 0x128;
template <int CTRL>
__device__ __forceinline__ float dpp_move_f(float v) { return __int_as_float(dpp_move<CTRL>(__float_as_int(v))); }
template <int CTRL>
__device__ __forceinline__ double dpp_move_d(double v) {
    return __hiloint2double(dpp_move<CTRL>(__double2hiint(v)), dpp_move<CTRL>(__double2loint(v)));
}
// v of lane ^ 16 / lane ^ 32, as the pair (own half or row pair's first, the other one): with both
// operands the same register the swap leaves row r & ~1 (half 0) in one result and row r | 1
// (half 1) in the other, in every lane.
struct LanePair { int a, b; };
__device__ __forceinline__ LanePair rows_xor16(int v) {
    const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return LanePair{(int)r[0], (int)r[1]};
}
__device__ __forceinline__ LanePair halves_xor32(int v) {
    const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return LanePair{(int)r[0], (int)r[1]};
}
__device__ __forceinline__ float max_xor16(float v) {
    const LanePair r = rows_xor16(__float_as_int(v));
    return fmaxf(__int_as_float(r.a), __int_as_float(r.b));
}
__device__ __forceinline__ float max_xor32(float v) {
    const LanePair r = halves_xor32(__float_as_int(v));
    return fmaxf(__int_as_float(r.a), __int_as_float(r.b));
}
__device__ __forceinline__ float sum_xor16(float v) {
    const LanePair r = rows_xor16(__float_as_int(v));
    return __int_as_float(r.a) + __int_as_float(r.b);
}
__device__ __forceinline__ float sum_xor32(float v) {
    const LanePair r = halves_xor32(__float_as_int(v));
    return __int_as_float(r.a) + __int_as_float(r.b);
}
__device__ __forceinline__ double sum_xor16(double v) {
    const LanePair lo = rows_xor16(__double2loint(v)), hi = rows_xor16(__double2hiint(v));
    return __hiloint2double(hi.a, lo.a) + __hiloint2double(hi.b, lo.b);
}
__device__ __forceinline__ double sum_xor32(double v) {
    const LanePair lo = halves_xor32(__double2loint(v)), hi = halves_xor32(__double2hiint(v));
    return __hiloint2double(hi.a, lo.a) + __hiloint2double(hi.b, lo.b);
}

// Reductions over the 16 lanes that share lane / 16 (one "row" of the wavefront); every lane gets the result.
__device__ __forceinline__ float row16_max(float v) {
    v = fmaxf(v, dpp_move_f<kDppXor1>(v));
    v = fmaxf(v, dpp_move_f<kDppXor2>(v));
    v = fmaxf(v, dpp_move_f<kDppRor4>(v));
    v = fmaxf(v, dpp_move_f<kDppRor8>(v));
    return v;
}
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_move_f<kDppXor1>(v);
    v += dpp_move_f<kDppXor2>(v);
    v += dpp_move_f<kDppRor4>(v);
    v += dpp_move_f<kDppRor8>(v);
    return v;
}
__device__ __forceinline__ double row16_sum(double v) {
    v += dpp_move_d<kDppXor1>(v);
    v += dpp_move_d<kDppXor2>(v);
    v += dpp_move_d<kDppRor4>(v);
    v += dpp_move_d<kDppRor8>(v);
    return v;
}

// ... and over the whole wavefront.
__device__ __forceinline__ float wave_max(float v) { return max_xor32(max_xor16(row16_max(v))); }
__device__ __forceinline__ float wave_sum(float v) { return sum_xor32(sum_xor16(row16_sum(v))); }
__device__ __forceinline__ double wave_sum(double v) { return sum_xor32(sum_xor16(row16_sum(v))); }

// Workgroup reductions for NW wavefronts; `red` is LDS scratch of at least NW floats.  Every
// thread of the workgroup must call; every thread gets the result.
template <int NW>
__device__ __forceinline__ float block_max(float v, float* red) {
    v = wave_max(v);
    if (NW == 1) return v;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) r = fmaxf(r, red[i]);
    return r;
}
template <int NW>
__device__ __forceinline__ float block_sum(float v, float* red) {
    v = wave_sum(v);
    if (NW == 1) return v;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) r += red[i];
    return r;
}

// The query-similarity test of Section 2.2 ("deciding when to decode with the full cache"): cosine
// similarity between the query of sequence b averaged over its Hq heads and the reference
// q_ref[b, :] kept from the last full step.  The work of one wavefront, in two parts, so that a
// kernel with other work can put the requests early and the arithmetic where it waits anyway.
// Lane (hg, dc) = (lane / 16, lane % 16) has dimensions 8 dc .. 8 dc + 7 of the heads hg, hg + 4,
// hg + 8, ...: one 16-byte load per lane fetches four whole heads per instruction.  The order of
// the fp32 additions is fixed: the heads of a lane group in order, then (group 0 + 1) + (2 + 3);
// the dot product and the two norms over a lane's 8 dimensions in order, then over the 16 lanes.
constexpr int kSimRound = 8;                      // loads per lane in flight together: 32 heads
struct SimLoads { uint4 v[kSimRound]; float4 r0, r1; };
// Part 1: requests the reference and the first 32 heads (one memory round trip).  q and q_ref are
// 16-byte aligned.
__device__ __forceinline__ void similarity_request(const uint16_t* q, const float* q_ref, int b, int Hq, SimLoads& ld) {
    const int lane = threadIdx.x & 63, hg = lane >> 4, dc = lane & 15;
    const float4* rp = reinterpret_cast<const float4*>(q_ref + (int64_t)b * RK_HEAD_DIM + dc * 8);
    ld.r0 = rp[0]; ld.r1 = rp[1];
    const uint16_t* qb = q + (int64_t)b * Hq * RK_HEAD_DIM + dc * 8;
#pragma unroll
    for (int i = 0; i < kSimRound; ++i)
        ld.v[i] = *reinterpret_cast<const uint4*>(qb + (int64_t)min(4 * i + hg, Hq - 1) * RK_HEAD_DIM);
}
// Part 2: the similarity, the same bits in every lane of every wavefront that computes it; mean[j]
// = component 8 dc + j of the averaged query (the same in the four lane groups).
__device__ __forceinline__ float similarity_finish(const uint16_t* q, int b, int Hq, const SimLoads& ld, float (&mean)[8]) {
    const int lane = threadIdx.x & 63, hg = lane >> 4, dc = lane & 15;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    auto add_head = [&](const uint4 x) {
        acc[0] += __uint_as_float(x.x << 16); acc[1] += __uint_as_float(x.x & 0xFFFF0000u);
        acc[2] += __uint_as_float(x.y << 16); acc[3] += __uint_as_float(x.y & 0xFFFF0000u);
        acc[4] += __uint_as_float(x.z << 16); acc[5] += __uint_as_float(x.z & 0xFFFF0000u);
        acc[6] += __uint_as_float(x.w << 16); acc[7] += __uint_as_float(x.w & 0xFFFF0000u);
    };
#pragma unroll
    for (int i = 0; i < kSimRound; ++i)
        if (4 * i + hg < Hq) add_head(ld.v[i]);
    const uint16_t* qb = q + (int64_t)b * Hq * RK_HEAD_DIM + dc * 8;
    for (int h0 = 4 * kSimRound; h0 < Hq; h0 += 4 * kSimRound) {      // more heads than one round holds
        uint4 v[kSimRound];
#pragma unroll
        for (int i = 0; i < kSimRound; ++i)
            v[i] = *reinterpret_cast<const uint4*>(qb + (int64_t)min(h0 + 4 * i + hg, Hq - 1) * RK_HEAD_DIM);
#pragma unroll
        for (int i = 0; i < kSimRound; ++i)
            if (h0 + 4 * i + hg < Hq) add_head(v[i]);
    }
    const float ref[8] = {ld.r0.x, ld.r0.y, ld.r0.z, ld.r0.w, ld.r1.x, ld.r1.y, ld.r1.z, ld.r1.w};
    float dot = 0.f, n1 = 0.f, n2 = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        mean[j] = sum_xor32(sum_xor16(acc[j])) / (float)Hq;
        dot += mean[j] * ref[j]; n1 += mean[j] * mean[j]; n2 += ref[j] * ref[j];
    }
    // (the lanes of a row of 16 add in different orders: lane 0 speaks for all)
    dot = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(row16_sum(dot))));
    n1 = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(row16_sum(n1))));
    n2 = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(row16_sum(n2))));
    return dot / (fmaxf(sqrtf(n1), 1e-8f) * fmaxf(sqrtf(n2), 1e-8f));
}

// fp64 sum over the workgroup; `red` holds NW doubles.
template <int NW>
__device__ __forceinline__ double block_sum_f64(double v, double* red) {
    v = wave_sum(v);
    if (NW == 1) return v;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = red[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) r += red[i];
    return r;
}

// Order-preserving map float -> uint32 (larger float <=> larger key) and its inverse.
__device__ __forceinline__ uint32_t key_of(float x) {
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float value_of(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}
// One step of the aggregation of the attention weights across the query heads of a GQA group
// (Section 2.2 footnote: max; Appendix A.3 also tries the mean and the group's first head).
// `acc` starts at -inf; head 0 always replaces it.  The mean is finished by a division by G.
__device__ __forceinline__ float aggregate(float acc, float w, int head, int agg) {
    if (head == 0) return w;
    if (agg == 0) return fmaxf(acc, w);       // RK_AGG_MAX
    if (agg == 1) return acc + w;             // RK_AGG_MEAN: heads added in order, in fp32
    return acc;                               // RK_AGG_FIRST
}

// Orders LDS traffic of the lanes of one wavefront: what was written before is visible to
// every lane after.  Lanes of a wavefront run in lockstep, so no hardware barrier is needed,
// only the compiler and the LDS queue have to be told.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace rk
