// The non-linear block of an LSTM cell (Section 2: slicing and element-wise operations on the two
// fully-connected outputs and the previous cell state), forward and backward, with the activations either
// recomputed in the backward pass from the kept sum a = Gx + Gh (Section 3.4) or read back from a stash
// (comparison).  Every kernel is a pure stream: per element of [B, H] the recompute path moves 60 bytes
// forward and 48 backward, the stash path 64 and 52, so they are bound by HBM bandwidth and the recompute
// path is the cheaper one in both footprint and traffic.
//
// A lane owns V consecutive hidden units of one row (V = 4: 16-byte loads and stores of each gate slice).
#include "../../include/echolstm.h"

#include <hip/hip_runtime.h>

#include "common.hpp"

namespace echo {

constexpr float kLog2eL = 1.4426950408889634f;

// sigmoid(x) = 1 / (1 + 2^(-x log2 e)); exp2 overflows to +inf for very negative x and the reciprocal gives 0.
__device__ __forceinline__ float sigmoid_f(float x) { return fast_rcp(1.0f + fast_exp2(-kLog2eL * x)); }
// tanh(x) = 1 - 2 / (2^(2 x log2 e) + 1); saturates to +-1 through the same overflow.
__device__ __forceinline__ float tanh_f(float x) {
    return __builtin_fmaf(-2.0f, fast_rcp(fast_exp2(kTwoLog2e * x) + 1.0f), 1.0f);
}

template <int V> struct Vec;
template <> struct Vec<4> {
    float v[4];
    __device__ __forceinline__ static Vec load(const float *p) {
        const float4 t = load4_streaming(p);   // plain loads measured 10 % slower at 16384 x 1024
        return Vec{{t.x, t.y, t.z, t.w}};
    }
    __device__ __forceinline__ void store(float *p) const { store4_streaming(p, make_float4(v[0], v[1], v[2], v[3])); }
};
template <> struct Vec<1> {
    float v[1];
    __device__ __forceinline__ static Vec load(const float *p) { return Vec{{*p}}; }
    __device__ __forceinline__ void store(float *p) const { store_streaming(p, v[0]); }
};

// STASH = false: writes h, c and the sum a.   STASH = true: writes h, c, the activations and tanh(c).
// a may alias Gx or Gh, so these three carry no __restrict__.
template <int V, bool STASH>
__global__ __launch_bounds__(256) void k_lstm_fwd(const float *Gx, const float *Gh,
                                                  const float *__restrict__ c_prev, float *__restrict__ h,
                                                  float *__restrict__ c, float *a_or_acts,
                                                  float *__restrict__ tanh_c, size_t H, size_t per_row,
                                                  size_t n_items) {
    const size_t it = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (it < n_items) {
        const size_t b = it / per_row, k = (it - b * per_row) * V;
        const size_t g0 = b * 4 * H + k, s0 = b * H + k;
        Vec<V> x[4], y[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            x[s] = Vec<V>::load(Gx + g0 + s * H);
            y[s] = Vec<V>::load(Gh + g0 + s * H);
        }
        const Vec<V> cp = Vec<V>::load(c_prev + s0);
        Vec<V> out[4], hv, cv, tv;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const float ai = x[0].v[e] + y[0].v[e], af = x[1].v[e] + y[1].v[e];
            const float ag = x[2].v[e] + y[2].v[e], ao = x[3].v[e] + y[3].v[e];
            const float i = sigmoid_f(ai), f = sigmoid_f(af), g = tanh_f(ag), o = sigmoid_f(ao);
            const float cc = __builtin_fmaf(f, cp.v[e], i * g);
            const float tc = tanh_f(cc);
            cv.v[e] = cc;
            hv.v[e] = o * tc;
            tv.v[e] = tc;
            out[0].v[e] = STASH ? i : ai;
            out[1].v[e] = STASH ? f : af;
            out[2].v[e] = STASH ? g : ag;
            out[3].v[e] = STASH ? o : ao;
        }
        hv.store(h + s0);
        cv.store(c + s0);
#pragma unroll
        for (int s = 0; s < 4; ++s) out[s].store(a_or_acts + g0 + s * H);
        if (STASH) tv.store(tanh_c + s0);
    }
}

// STASH = false: src = a, the activations and tanh(c) are re-evaluated.  STASH = true: src = acts, tanh_c read.
template <int V, bool STASH>
__global__ __launch_bounds__(256) void k_lstm_bwd(const float *__restrict__ dh, const float *__restrict__ dc,
                                                  const float *__restrict__ src,
                                                  const float *__restrict__ tanh_c,
                                                  const float *__restrict__ c_prev, float *__restrict__ da,
                                                  float *__restrict__ dc_prev, size_t H, size_t per_row,
                                                  size_t n_items) {
    const size_t it = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (it < n_items) {
        const size_t b = it / per_row, k = (it - b * per_row) * V;
        const size_t g0 = b * 4 * H + k, s0 = b * H + k;
        Vec<V> x[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) x[s] = Vec<V>::load(src + g0 + s * H);
        const Vec<V> cp = Vec<V>::load(c_prev + s0);
        const Vec<V> gh = Vec<V>::load(dh + s0);
        Vec<V> gc, tv;
        if (dc) gc = Vec<V>::load(dc + s0);
        if (STASH) tv = Vec<V>::load(tanh_c + s0);
        Vec<V> out[4], dcp;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            float i, f, g, o, tc;
            if (STASH) {
                i = x[0].v[e], f = x[1].v[e], g = x[2].v[e], o = x[3].v[e], tc = tv.v[e];
            } else {
                i = sigmoid_f(x[0].v[e]), f = sigmoid_f(x[1].v[e]), g = tanh_f(x[2].v[e]), o = sigmoid_f(x[3].v[e]);
                tc = tanh_f(__builtin_fmaf(f, cp.v[e], i * g));
            }
            const float d_h = gh.v[e];
            const float d_o = d_h * tc;
            const float dct = __builtin_fmaf(d_h * o, 1.0f - tc * tc, dc ? gc.v[e] : 0.0f);
            dcp.v[e] = dct * f;
            out[0].v[e] = dct * g * (i * (1.0f - i));
            out[1].v[e] = dct * cp.v[e] * (f * (1.0f - f));
            out[2].v[e] = dct * i * (1.0f - g * g);
            out[3].v[e] = d_o * (o * (1.0f - o));
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) out[s].store(da + g0 + s * H);
        dcp.store(dc_prev + s0);
    }
}

// One cell of the translation model is only a few thousand items: single-wave blocks then reach every CU.
static int lstm_threads(size_t n_items) { return n_items <= 64 * 1024 ? 64 : 256; }
// One item per thread, blocks in address order (a fixed grid of 4096 blocks striding over the arrays measured
// 2 to 5 % slower at 16384 x 1024).  check_shape keeps the block count below 2^31.
static unsigned lstm_grid(size_t n_items) {
    const size_t t = lstm_threads(n_items);
    return (unsigned)((n_items + t - 1) / t);
}

static bool misaligned(std::initializer_list<const void *> ps) {
    uintptr_t m = 0;
    for (const void *p : ps) m |= (uintptr_t)p;
    return (m & 15u) != 0;
}

static echo_status_t check_shape(int64_t B, int64_t H) {
    if (B < 1 || H < 1) return ECHO_ERR_SHAPE;
    if (H > (int64_t(1) << 38) || B > (int64_t(1) << 38) / H) return ECHO_ERR_SHAPE;
    return ECHO_OK;
}

template <bool STASH>
static echo_status_t fwd_impl(int64_t B, int64_t H, const float *Gx, const float *Gh, const float *c_prev, float *h,
                              float *c, float *a_or_acts, float *tanh_c, void *stream) {
    if (!Gx || !Gh || !c_prev || !h || !c || !a_or_acts || (STASH && !tanh_c)) return ECHO_ERR_NULL;
    if (echo_status_t s = check_shape(B, H)) return s;
    if (misaligned({Gx, Gh, c_prev, h, c, a_or_acts, tanh_c})) return ECHO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (H % 4 == 0) {
        const size_t per_row = H / 4, n = (size_t)B * per_row;
        k_lstm_fwd<4, STASH><<<lstm_grid(n), lstm_threads(n), 0, st>>>(Gx, Gh, c_prev, h, c, a_or_acts, tanh_c, H, per_row, n);
    } else {
        const size_t n = (size_t)B * H;
        k_lstm_fwd<1, STASH><<<lstm_grid(n), lstm_threads(n), 0, st>>>(Gx, Gh, c_prev, h, c, a_or_acts, tanh_c, H, H, n);
    }
    return hipGetLastError() == hipSuccess ? ECHO_OK : ECHO_ERR_HIP;
}

template <bool STASH>
static echo_status_t bwd_impl(int64_t B, int64_t H, const float *dh, const float *dc, const float *src,
                              const float *tanh_c, const float *c_prev, float *da, float *dc_prev, void *stream) {
    if (!dh || !src || !c_prev || !da || !dc_prev || (STASH && !tanh_c)) return ECHO_ERR_NULL;
    if (echo_status_t s = check_shape(B, H)) return s;
    if (misaligned({dh, dc, src, tanh_c, c_prev, da, dc_prev})) return ECHO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (H % 4 == 0) {
        const size_t per_row = H / 4, n = (size_t)B * per_row;
        k_lstm_bwd<4, STASH><<<lstm_grid(n), lstm_threads(n), 0, st>>>(dh, dc, src, tanh_c, c_prev, da, dc_prev, H, per_row, n);
    } else {
        const size_t n = (size_t)B * H;
        k_lstm_bwd<1, STASH><<<lstm_grid(n), lstm_threads(n), 0, st>>>(dh, dc, src, tanh_c, c_prev, da, dc_prev, H, H, n);
    }
    return hipGetLastError() == hipSuccess ? ECHO_OK : ECHO_ERR_HIP;
}

}  // namespace echo

extern "C" {

echo_status_t echo_lstm_cell_fwd(int64_t B, int64_t H, const float *Gx, const float *Gh, const float *c_prev,
                                 float *h, float *c, float *a, void *stream) {
    return echo::fwd_impl<false>(B, H, Gx, Gh, c_prev, h, c, a, nullptr, stream);
}

echo_status_t echo_lstm_cell_bwd(int64_t B, int64_t H, const float *dh, const float *dc, const float *a,
                                 const float *c_prev, float *da, float *dc_prev, void *stream) {
    return echo::bwd_impl<false>(B, H, dh, dc, a, nullptr, c_prev, da, dc_prev, stream);
}

echo_status_t echo_lstm_cell_fwd_stash(int64_t B, int64_t H, const float *Gx, const float *Gh,
                                       const float *c_prev, float *h, float *c, float *acts, float *tanh_c,
                                       void *stream) {
    return echo::fwd_impl<true>(B, H, Gx, Gh, c_prev, h, c, acts, tanh_c, stream);
}

echo_status_t echo_lstm_cell_bwd_stash(int64_t B, int64_t H, const float *dh, const float *dc,
                                       const float *acts, const float *tanh_c, const float *c_prev, float *da,
                                       float *dc_prev, void *stream) {
    return echo::bwd_impl<true>(B, H, dh, dc, acts, tanh_c, c_prev, da, dc_prev, stream);
}

size_t echo_lstm_cell_kept_bytes(int64_t B, int64_t H, int stash) {
    if (B < 1 || H < 1) return 0;
    return (size_t)(stash ? 6 : 5) * (size_t)B * (size_t)H * sizeof(float);
}

}  // extern "C"
