// Measurement support: synthetic kernels that issue one class of vector
// instruction (or the instruction mix of the two hot loops) on every CU, and a
// plain copy, so the benchmark can state the ceilings it measures against.
#include "../../include/echoattn.h"
#include "common.hpp"

namespace echo {

constexpr int CAL_CHAINS = 16;     // independent dependency chains per lane
constexpr int CAL_UNROLL = 8;      // instructions per chain and loop trip

template <int KIND>
__global__ __launch_bounds__(256) void k_cal_alu(float *__restrict__ out, int iters, float seed) {
    float x[CAL_CHAINS];
    const float a = 0.999f + seed * 1e-6f, c = seed * 1e-7f;
#pragma unroll
    for (int k = 0; k < CAL_CHAINS; ++k) x[k] = seed + 0.01f * (float)(k + 1) + 1e-3f * (float)(threadIdx.x & 63);
    float accA = 0.f, accB = 0.f, accC = 0.f;
    float aa = a;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < CAL_UNROLL; ++u) {
            aa += c;                      // keeps the mixes from being hoisted; 1 op per 16 chains
#pragma unroll
            for (int k = 0; k < CAL_CHAINS; ++k) {
                if (KIND == ECHO_CAL_FMA) {
                    x[k] = __builtin_fmaf(x[k], a, c);
                } else if (KIND == ECHO_CAL_RCP) {
                    x[k] = fast_rcp(x[k]);
                } else if (KIND == ECHO_CAL_EXP2) {
                    x[k] = fast_exp2(x[k]);
                } else if (KIND == ECHO_CAL_FWD_MIX) {          // fma, rcp, fma: one tanh of the score loop
                    const float r = fast_rcp(__builtin_fmaf(x[k], aa, 1.0f));
                    accA = __builtin_fmaf(c, r, accA);
                } else {                                        // fma, rcp, 4 fma: one tanh of the recompute loop
                    const float r = fast_rcp(__builtin_fmaf(x[k], aa, 1.0f));
                    const float w = __builtin_fmaf(-r, r, r);
                    accA = __builtin_fmaf(c, w, accA);
                    accB = __builtin_fmaf(a, w, accB);
                    accC = __builtin_fmaf(c, r, accC);
                }
            }
        }
    }
    float s = accA + accB + accC;
#pragma unroll
    for (int k = 0; k < CAL_CHAINS; ++k) s += x[k];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void k_cal_copy(const float4 *__restrict__ src, float4 *__restrict__ dst, size_t n4) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride)
        store4_streaming(reinterpret_cast<float *>(dst + i), src[i]);
}

}  // namespace echo

extern "C" echo_status_t echo_attn_calibrate(int kind, int blocks, int iters, const void *src, void *dst,
                                             size_t bytes, double *work, void *stream) {
    using namespace echo;
    if (!dst || !work) return ECHO_ERR_NULL;
    if (blocks < 1 || iters < 1) return ECHO_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(dst) & 15u) || (reinterpret_cast<uintptr_t>(src) & 15u)) return ECHO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    float *out = static_cast<float *>(dst);
    if (kind != ECHO_CAL_COPY && bytes < (size_t)blocks * 256 * sizeof(float)) return ECHO_ERR_WORKSPACE;
    const double per_lane = (double)iters * CAL_UNROLL * CAL_CHAINS;
    const double lanes = (double)blocks * 256;
    switch (kind) {
        case ECHO_CAL_FMA: k_cal_alu<ECHO_CAL_FMA><<<blocks, 256, 0, st>>>(out, iters, 1.0f); break;
        case ECHO_CAL_RCP: k_cal_alu<ECHO_CAL_RCP><<<blocks, 256, 0, st>>>(out, iters, 1.0f); break;
        case ECHO_CAL_EXP2: k_cal_alu<ECHO_CAL_EXP2><<<blocks, 256, 0, st>>>(out, iters, -1.0f); break;
        case ECHO_CAL_FWD_MIX: k_cal_alu<ECHO_CAL_FWD_MIX><<<blocks, 256, 0, st>>>(out, iters, 1.0f); break;
        case ECHO_CAL_BWD_MIX: k_cal_alu<ECHO_CAL_BWD_MIX><<<blocks, 256, 0, st>>>(out, iters, 1.0f); break;
        case ECHO_CAL_COPY:
            if (!src) return ECHO_ERR_NULL;
            if (bytes < 16) return ECHO_ERR_SHAPE;
            k_cal_copy<<<blocks, 256, 0, st>>>(static_cast<const float4 *>(src), static_cast<float4 *>(dst), bytes / 16);
            *work = (double)(bytes / 16 * 16);
            return hipGetLastError() == hipSuccess ? ECHO_OK : ECHO_ERR_HIP;
        default: return ECHO_ERR_DTYPE;
    }
    *work = per_lane * lanes;
    return hipGetLastError() == hipSuccess ? ECHO_OK : ECHO_ERR_HIP;
}
