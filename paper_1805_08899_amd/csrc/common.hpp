// Device helpers shared by the libechoattn kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace echo {

// bf16 storage: the upper 16 bits of an IEEE float.
struct bf16_t { uint16_t bits; };

template <typename T> __device__ __forceinline__ float ld(const T *p, size_t i);
template <> __device__ __forceinline__ float ld<float>(const float *p, size_t i) { return p[i]; }
template <> __device__ __forceinline__ float ld<bf16_t>(const bf16_t *p, size_t i) {
    return __uint_as_float(static_cast<uint32_t>(p[i].bits) << 16);
}

// Four consecutive elements starting at a multiple of four (16-byte / 8-byte aligned).
__device__ __forceinline__ float4 ld4(const float *p, size_t i) {
    return *reinterpret_cast<const float4 *>(p + i);
}
__device__ __forceinline__ float4 ld4(const bf16_t *p, size_t i) {
    uint2 u = *reinterpret_cast<const uint2 *>(p + i);
    float4 r;
    r.x = __uint_as_float(u.x << 16);
    r.y = __uint_as_float(u.x & 0xffff0000u);
    r.z = __uint_as_float(u.y << 16);
    r.w = __uint_as_float(u.y & 0xffff0000u);
    return r;
}

// tanh(x) = 1 - 2 / (exp(2x) + 1).  With s = 2*log2(e)*x this is
// 1 - 2*rcp(exp2(s) + 1); exp2 -> inf gives 1, exp2 -> 0 gives -1, no NaN.
constexpr float kTwoLog2e = 2.8853900817779268f;

// exp(2(q+k)) = exp(2q) * exp(2k): the exponentials are taken once per row
// element and the inner loop needs one multiply-add and one reciprocal.  The
// factors stay finite and normal while |x| <= kFactorLimit (|s| <= 115.4), and
// their product then overflows to inf or underflows to 0 exactly where tanh
// has saturated, never to NaN.  Rows with a larger |x| take the exact path,
// which exponentiates the sum.
constexpr float kFactorLimit = 40.0f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

// r = 1 / (exp(2x) + 1) from the two factors:  tanh = 1 - 2r,  1 - tanh^2 = 4 r (1 - r).
__device__ __forceinline__ float r_from_factors(float eq, float ek) {
    return fast_rcp(__builtin_fmaf(eq, ek, 1.0f));
}
// same from the scaled pre-activations sq = c*q, sk = c*k (exact path)
__device__ __forceinline__ float r_from_sum(float sq, float sk) {
    return fast_rcp(fast_exp2(sq + sk) + 1.0f);
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); }

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}

// Sum N per-lane arrays over the 64 lanes of a wave at a cost of about one
// exchange per value instead of six: at each butterfly level a lane keeps one
// half of its values and hands the other half to its partner.  On return lane
// l holds in a[0] the full sum of value number (l mod N).  N is a power of two
// <= 64; the order of additions is fixed.
template <int N, int OFF>
struct TransposeSumStep {
    // N values are still spread over lanes whose index differs in bit OFF and below
    template <int M>
    static __device__ __forceinline__ void run(float (&a)[M], int lane) {
        if constexpr (OFF >= N) {   // more lanes than values left to split: plain butterfly
#pragma unroll
            for (int k = 0; k < N; ++k) a[k] += __shfl_xor(a[k], OFF, 64);
            if constexpr (OFF > 1) TransposeSumStep<N, OFF / 2>::run(a, lane);
        } else {
            const bool hi = (lane & OFF) != 0;
            constexpr int half = N / 2;
#pragma unroll
            for (int k = 0; k < half; ++k) {
                const float keep = hi ? a[k + half] : a[k];
                const float send = hi ? a[k] : a[k + half];
                a[k] = keep + __shfl_xor(send, OFF, 64);
            }
            if constexpr (OFF > 1) TransposeSumStep<half, OFF / 2>::run(a, lane);
        }
    }
};

template <int N>
__device__ __forceinline__ float wave_transpose_sum(float (&a)[N]) {
    static_assert(N >= 1 && N <= 64 && (N & (N - 1)) == 0, "N must be a power of two <= 64");
    TransposeSumStep<N, 32>::run(a, lane_id());
    return a[0];
}

__device__ __forceinline__ int clamp_len(int len, int Tk) { return len < 0 ? 0 : (len > Tk ? Tk : len); }

}  // namespace echo
