// F2: masked softmax over the keys of one (b, i) row (attention weights,
// Section 2 step 1), and B4: the fixed-order reduction that finishes dv.
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

// dv[h] = c0 + sum_b dv_part[b,h];  c0 = sum over all rows of ds_rowsum (the
// part of sum dS*tanh that comes from tanh = 1 - 2r; it is zero in exact
// arithmetic because every row of dS sums to zero).  Block = 64 values of h x
// 4 groups of samples; every partial sum and the final combination run in a
// fixed order, so the result is reproducible.
__global__ __launch_bounds__(256) void k_dv_reduce(const float *__restrict__ dv_part,
                                                  const float *__restrict__ ds_rowsum, float *__restrict__ dv,
                                                  int B, int rows, int H) {
    __shared__ float s_c0[256];
    __shared__ float s_acc[4][64];
    const int lane = lane_id(), g = wave_id();
    // loads go out eight at a time so that their latencies overlap
    float c0 = 0.f;
    for (int r0 = threadIdx.x; r0 < rows; r0 += 8 * 256) {
        float x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = (r0 + u * 256 < rows) ? ds_rowsum[r0 + u * 256] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) c0 += x[u];
    }
    s_c0[threadIdx.x] = c0;
    const int h = blockIdx.x * 64 + lane;
    float acc = 0.f;
    if (h < H) {
        for (int b0 = g; b0 < B; b0 += 8 * 4) {
            float x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = (b0 + 4 * u < B) ? dv_part[(size_t)(b0 + 4 * u) * H + h] : 0.f;
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += x[u];
        }
    }
    s_acc[g][lane] = acc;
    __syncthreads();
    if (g == 0) {
        float c = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) c += s_c0[lane + 64 * k];
        c = wave_sum(c);
        if (h < H) dv[h] = ((s_acc[0][lane] + s_acc[1][lane]) + (s_acc[2][lane] + s_acc[3][lane])) + c;
    }
}

hipError_t launch_dv_reduce(const AttnShape &s, const float *dv_part, const float *ds_rowsum, float *dv,
                            hipStream_t st) {
    k_dv_reduce<<<(s.H + 63) / 64, 256, 0, st>>>(dv_part, ds_rowsum, dv, s.B, s.B * s.Tq, s.H);
    return hipGetLastError();
}

}  // namespace echo
