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

// Non-temporal loads, for inputs read once by the whole grid.  Measured: they help the LSTM block (nine input and
// output streams at once, 180 -> 170 us) and hurt a single-stream copy (76 -> 93 us), so only the former uses them
// (in the recompute kernel they cost 1 to 8 %).
__device__ __forceinline__ float4 load4_streaming(const float *p) {
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4 v = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
// Stores of results that this kernel does not read again go out as non-temporal (streaming) stores: they do not
// stay behind as dirty lines for the end of the kernel to write back, which measured 0.3 to 0.6 us per kernel at
// the smallest benchmark workload and 5 % of a pure streaming kernel.
__device__ __forceinline__ void store_streaming(float *p, float x) { __builtin_nontemporal_store(x, p); }
__device__ __forceinline__ void store4_streaming(float *p, float4 x) {
    typedef float f4 __attribute__((ext_vector_type(4)));
    __builtin_nontemporal_store((f4){x.x, x.y, x.z, x.w}, reinterpret_cast<f4 *>(p));
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

// Reductions over the 64 lanes, result in every lane.  Within a row of 16 lanes the partners are reached with DPP
// (two quad permutations, then the two mirror patterns); the four row results are then read as scalars.  A dozen
// full-rate instructions, where six general shuffles would each take a trip through the LDS crossbar.
template <int CTRL> __device__ __forceinline__ float dpp_get(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}
template <int CTRL> __device__ __forceinline__ uint32_t dpp_get_u32(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, false);
}
__device__ __forceinline__ float lane_value(float x, int l) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), l));
}
__device__ __forceinline__ float wave_sum(float x) {
    x += dpp_get<0xB1>(x);      // quad_perm [1,0,3,2]
    x += dpp_get<0x4E>(x);      // quad_perm [2,3,0,1]
    x += dpp_get<0x141>(x);     // row_half_mirror
    x += dpp_get<0x140>(x);     // row_mirror
    return (lane_value(x, 0) + lane_value(x, 16)) + (lane_value(x, 32) + lane_value(x, 48));
}
__device__ __forceinline__ float wave_max(float x) {
    x = fmaxf(x, dpp_get<0xB1>(x));
    x = fmaxf(x, dpp_get<0x4E>(x));
    x = fmaxf(x, dpp_get<0x141>(x));
    x = fmaxf(x, dpp_get<0x140>(x));
    return fmaxf(fmaxf(lane_value(x, 0), lane_value(x, 16)), fmaxf(lane_value(x, 32), lane_value(x, 48)));
}

// ---------------------------------------------------------------------------
// Sum N per-lane arrays over the 64 lanes of a wave at a cost of about one
// exchange per value instead of six.  At each level a lane keeps one half of
// its values and hands the other half to the partner lane `OFF` away (levels
// 32 and 16 with the gfx950 lane-swap instructions, 8 and 4 with DPP row
// shifts selected by bank masks, 2 and 1 with quad permutations); once one value is left the group of
// lanes that shares it is summed with quad permutations and the two mirror patterns (and, for N < 8, lane swaps
// of a value with itself).  On return lane l holds in a[0] the full sum of value
// number l / (64 / N).  N is a power of two <= 64; the order of additions is fixed.
template <int CTRL, int BANK_MASK, bool BOUND>
__device__ __forceinline__ float dpp_mov(float old, float src) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(src), CTRL, 0xf, BANK_MASK, BOUND));
}

// x = value kept by lanes whose bit OFF is 0, y = value kept by the others.
template <int OFF>
__device__ __forceinline__ float transpose_pair(float x, float y, int lane) {
    if constexpr (OFF == 32) {
        auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(y), false, false);
        return __uint_as_float(r[0]) + __uint_as_float(r[1]);
    } else if constexpr (OFF == 16) {
        auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(y), false, false);
        return __uint_as_float(r[0]) + __uint_as_float(r[1]);
    } else if constexpr (OFF == 8 || OFF == 4) {
        constexpr int SHL = 0x100 + OFF, SHR = 0x110 + OFF;     // row_shl:OFF / row_shr:OFF
        constexpr int LO_BANKS = OFF == 8 ? 0x3 : 0x5;           // lanes of a row whose bit OFF is 0
        const float t_lo = x + dpp_mov<SHL, 0xf, true>(0.f, x);  // x[l] + x[l + OFF]   (right where bit OFF is 0)
        const float t_hi = y + dpp_mov<SHR, 0xf, true>(0.f, y);  // y[l] + y[l - OFF]   (right where bit OFF is 1)
        return dpp_mov<0xE4, LO_BANKS, false>(t_hi, t_lo);       // identity move into the low banks only
    } else {                                                     // partner inside the quad: one quad permutation
        static_assert(OFF == 2 || OFF == 1, "lane offsets are powers of two below 64");
        const bool hi = (lane & OFF) != 0;
        const float keep = hi ? y : x;
        const float send = hi ? x : y;
        return keep + dpp_get<OFF == 2 ? 0x4E : 0xB1>(send);
    }
}

template <int N, int OFF>
struct TransposeSumStep {
    template <int M>
    static __device__ __forceinline__ void run(float (&a)[M], int lane) {
        if constexpr (N == 1) {      // one value left: sum over the group of 2 OFF lanes that share it
            a[0] += dpp_get<0xB1>(a[0]);                              // lanes l ^ 1
            if constexpr (OFF >= 2) a[0] += dpp_get<0x4E>(a[0]);      // l ^ 2: the quad
            if constexpr (OFF >= 4) a[0] += dpp_get<0x141>(a[0]);     // mirror in the half row: the other quad
            if constexpr (OFF >= 8) a[0] += dpp_get<0x140>(a[0]);     // mirror in the row: the other half
            if constexpr (OFF >= 16) a[0] = transpose_pair<16>(a[0], a[0], lane);   // the neighbouring row
            if constexpr (OFF >= 32) a[0] = transpose_pair<32>(a[0], a[0], lane);   // the other half of the wave
        } else {
            constexpr int half = N / 2;
#pragma unroll
            for (int k = 0; k < half; ++k) a[k] = transpose_pair<OFF>(a[k], a[k + half], lane);
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

// Barrier for data exchanged through LDS only: waits for this wave's LDS operations, not for its global
// loads and stores (__syncthreads() would also wait for every prefetch and store in flight).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Accesses that other blocks of the same launch must see (or that must see theirs): device-scope relaxed
// atomics, which go through to the memory side of the per-XCD L2 caches instead of staying in one of them.
// Ordering between them is the program order of the issuing wave plus an explicit wait on the memory counter.
__device__ __forceinline__ void store_agent(float *p, float x) {
    __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_agent(const float *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_agent(unsigned long long *p, unsigned long long x) {
    __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long load_agent(const unsigned long long *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void wait_all_memory_ops() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// A wait on another block's flag gives up after this many ticks of the 100 MHz wall clock (2 s), so that every
// wave ends whatever happens; the results of that launch are then marked invalid (NaN).
constexpr long long kSpinLimitTicks = 200000000LL;

__device__ __forceinline__ int clamp_len(int len, int Tk) { return len < 0 ? 0 : (len > Tk ? Tk : len); }

// n items dealt to the 8 waves of a block as contiguous ranges of n / 8 or n / 8 + 1 items: first item of wave w
// (w = 8 gives n).  Waves w and w + 4 run on the same SIMD, so the n % 8 longer ranges go to waves
// 0, 5, 2, 7, 4, 1, 6, 3 in that order: the SIMDs' totals then differ by at most one item, where the plain
// floor(n w / 8) split would hand both longer ranges of n % 8 == 2 to one SIMD.
__device__ __forceinline__ int deal8_begin(int n, int w) {
    // byte e: bit w set if wave w gets a longer range when n % 8 == e (0x00, 0x01, 0x21, 0x25, 0xa5, 0xb5, 0xb7,
    // 0xf7).  Packed into one immediate: as an array the table sits in memory, and the scalar load that fetches
    // it is a trip to memory at the start of a block, right in front of the loads that depend on the ranges.
    constexpr unsigned long long kLonger = 0xf7b7b5a525210100ull;
    const unsigned m = (unsigned)(kLonger >> (8 * (n & 7))) & 0xffu;
    return (n >> 3) * w + __builtin_popcount(m & ((1u << w) - 1u));
}

}  // namespace echo
