// F2: masked softmax over the keys of one (b, i) row (attention weights,
// Section 2 step 1), used when the forward pass is not fused.
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

}  // namespace echo
