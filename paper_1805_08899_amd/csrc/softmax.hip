// F2: masked softmax over the keys of one (b, i) row (attention weights,
// Section 2 step 1), used when the forward pass is not fused; and B4: the
// fixed-order reduction that finishes dv.
#include "common.hpp"
#include "kernels.hpp"

namespace echo {

constexpr float kLog2e = 1.4426950408889634f;

// One wave per row.  Keys j >= L_b get probability exactly 0; a row with no
// valid key is all zeros.  The row maximum is subtracted before exponentiating.
__global__ __launch_bounds__(256) void k_softmax(const float *__restrict__ S, const int *__restrict__ key_len,
                                                 float *__restrict__ P, int rows, int Tq, int Tk) {
    const int row = blockIdx.x * 4 + wave_id();
    if (row >= rows) return;
    const int lane = lane_id();
    const int b = row / Tq;
    const int L = clamp_len(key_len[b], Tk);
    const float *s = S + (size_t)row * Tk;
    float *p = P + (size_t)row * Tk;
    float m = -INFINITY;
    for (int j = lane; j < L; j += 64) m = fmaxf(m, s[j]);
    m = wave_max(m);
    float z = 0.f;
    for (int j = lane; j < L; j += 64) z += fast_exp2((s[j] - m) * kLog2e);
    z = wave_sum(z);
    const float inv = 1.0f / z;
    for (int j = lane; j < Tk; j += 64) p[j] = j < L ? fast_exp2((s[j] - m) * kLog2e) * inv : 0.f;
}

hipError_t launch_softmax(const AttnShape &s, const float *S, const int *key_len, float *P, hipStream_t st) {
    const int rows = s.B * s.Tq;
    k_softmax<<<(rows + 3) / 4, 256, 0, st>>>(S, key_len, P, rows, s.Tq, s.Tk);
    return hipGetLastError();
}

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
