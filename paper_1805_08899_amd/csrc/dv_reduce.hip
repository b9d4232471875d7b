// B4 as a launch of its own: the fixed-order reduction that finishes dv after a sentence of decoder steps
// (echo_attn_step_finish).  The batched backward call does the same sum inside its recompute launch.
#include "common.hpp"
#include "kernels.hpp"

namespace echo {

// dv[h] = sum_b dv_part[b,h] (added to dv when add_to is set).  Block = 64 values of h x 8 groups of samples:
// group g adds samples g, g + 8, ... with eight loads in flight at a time, then
// the groups' sums are added in group order, so the result is reproducible.
__global__ __launch_bounds__(512) void k_dv_reduce(const float *__restrict__ dv_part, float *__restrict__ dv, int B,
                                                  int H, int add_to) {
    __shared__ float s_acc[8][64];
    const int lane = lane_id(), g = wave_id();
    const int h = blockIdx.x * 64 + lane;
    float acc = 0.f;
    if (h < H) {
        for (int b0 = g; b0 < B; b0 += 8 * 8) {
            float x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = (b0 + 8 * u < B) ? dv_part[(size_t)(b0 + 8 * u) * H + h] : 0.f;
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += x[u];
        }
    }
    s_acc[g][lane] = acc;
    __syncthreads();
    if (g == 0 && h < H) {
        float tot = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) tot += s_acc[k][lane];
        dv[h] = add_to ? dv[h] + tot : tot;
    }
}

hipError_t launch_dv_reduce(const AttnShape &s, const float *dv_part, float *dv, hipStream_t st) {
    k_dv_reduce<<<(s.H + 63) / 64, 512, 0, st>>>(dv_part, dv, s.B, s.H, s.acc ? 1 : 0);
    return hipGetLastError();
}

}  // namespace echo
