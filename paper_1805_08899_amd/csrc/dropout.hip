// Dropout with a one-bit feature map (Section 5.2: encode to 1 bit in the forward pass, decode back to 32 bits
// in the backward pass).  Both kernels are pure streams: the forward reads 4 bytes per element and writes
// 4 + 1/8, the backward reads 4 + 1/8 and writes 4, so they are bound by HBM bandwidth.
//
// A lane owns four consecutive elements (one 16-byte load and store, and exactly one Philox4x32-10 block);
// eight consecutive lanes own the 32 elements of one mask word and assemble it with three exchanges.
// The launch has one thread per four elements: blocks start in address order, so the blocks that run at any
// moment cover a narrow window of the arrays.  A fixed grid of 4096 blocks striding over the arrays measured
// 14 % slower (forward, 2^26 elements) and 20 % slower once the arrays no longer fit the on-die cache.
#include "../../include/echodropout.h"

#include <hip/hip_runtime.h>

#include "common.hpp"

namespace echo {

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC 2011): ten rounds of two 32x32 -> 64 bit multiplications
// and xors; the key is advanced by the two Weyl constants between rounds.
struct u32x4 { uint32_t x, y, z, w; };
__device__ __forceinline__ u32x4 philox4x32_10(u32x4 c, uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        if (r > 0) {
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        const uint64_t p0 = (uint64_t)0xD2511F53u * c.x, p1 = (uint64_t)0xCD9E8D57u * c.z;
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        c = u32x4{hi1 ^ c.y ^ k0, lo1, hi0 ^ c.w ^ k1, lo0};
    }
    return c;
}

__device__ __forceinline__ bool keep_from_word(uint32_t word, float p) {
    return static_cast<float>(word >> 8) * 5.9604644775390625e-08f >= p;   // (word >> 8) * 2^-24, exact in fp32
}

// Elements past n read as zero and are not written; their mask bits are zero.
__global__ __launch_bounds__(256) void k_dropout_fwd(const float *__restrict__ x, size_t n, float p, float scale,
                                                    uint32_t seed_lo, uint32_t seed_hi, uint32_t off_lo,
                                                    uint32_t off_hi, float *__restrict__ y,
                                                    uint32_t *__restrict__ mask_bits, size_t n_quads) {
    const int lane = lane_id();
    const size_t q = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (q < (n_quads + 7) / 8 * 8) {          // whole mask words: the eight lanes of a group stay together
        const size_t i = 4 * q;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i + 3 < n) v = *reinterpret_cast<const float4 *>(x + i);
        else if (i < n) {
            v.x = x[i];
            if (i + 1 < n) v.y = x[i + 1];
            if (i + 2 < n) v.z = x[i + 2];
        }
        const u32x4 r = philox4x32_10(u32x4{(uint32_t)q, (uint32_t)(q >> 32), off_lo, off_hi}, seed_lo, seed_hi);
        const bool k0 = i < n && keep_from_word(r.x, p), k1 = i + 1 < n && keep_from_word(r.y, p);
        const bool k2 = i + 2 < n && keep_from_word(r.z, p), k3 = i + 3 < n && keep_from_word(r.w, p);
        const float4 o = make_float4(k0 ? v.x * scale : 0.f, k1 ? v.y * scale : 0.f, k2 ? v.z * scale : 0.f,
                                     k3 ? v.w * scale : 0.f);
        if (i + 3 < n) store4_streaming(y + i, o);
        else if (i < n) {
            y[i] = o.x;
            if (i + 1 < n) y[i + 1] = o.y;
            if (i + 2 < n) y[i + 2] = o.z;
        }
        // this lane's four bits at their place in the word of its group of eight lanes, then OR over the group
        uint32_t bits = ((uint32_t)k0 | (uint32_t)k1 << 1 | (uint32_t)k2 << 2 | (uint32_t)k3 << 3) << (4 * (lane & 7));
        bits |= dpp_get_u32<0xB1>(bits);      // lanes l ^ 1 (quad permutation)
        bits |= dpp_get_u32<0x4E>(bits);      // l ^ 2: the quad holds its 16 bits
        bits |= dpp_get_u32<0x141>(bits);     // mirror in the half row: the other quad of the group of eight
        if ((lane & 7) == 0 && i < n) mask_bits[q / 8] = bits;
    }
}

__global__ __launch_bounds__(256) void k_dropout_bwd(const float *__restrict__ dy,
                                                    const uint32_t *__restrict__ mask_bits, size_t n, float scale,
                                                    float *__restrict__ dx, size_t n_quads) {
    const size_t q = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (q < n_quads) {
        const size_t i = 4 * q;
        // both loads leave before either is awaited (the eight lanes of a group share the mask word)
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i + 3 < n) v = *reinterpret_cast<const float4 *>(dy + i);
        else {
            v.x = dy[i];
            if (i + 1 < n) v.y = dy[i + 1];
            if (i + 2 < n) v.z = dy[i + 2];
        }
        const uint32_t bits = mask_bits[q / 8] >> (4 * (q & 7));
        const float4 o = make_float4((bits & 1u) ? v.x * scale : 0.f, (bits & 2u) ? v.y * scale : 0.f,
                                     (bits & 4u) ? v.z * scale : 0.f, (bits & 8u) ? v.w * scale : 0.f);
        if (i + 3 < n) store4_streaming(dx + i, o);
        else {
            dx[i] = o.x;
            if (i + 1 < n) dx[i + 1] = o.y;
            if (i + 2 < n) dx[i + 2] = o.z;
        }
    }
}

constexpr size_t kMaxElements = (size_t)1 << 40;      // 2^30 blocks of 256 quads
static unsigned stream_grid(size_t n_quads) { return (unsigned)((n_quads + 255) / 256); }

}  // namespace echo

extern "C" {

size_t echo_dropout_mask_words(size_t n) { return (n + 31) / 32; }

echo_status_t echo_dropout_fwd(const float *x, size_t n, float p, uint64_t seed, uint64_t offset, float *y,
                               uint32_t *mask_bits, void *stream) {
    if (!x || !y || !mask_bits) return ECHO_ERR_NULL;
    if (n == 0 || n > echo::kMaxElements || !(p >= 0.f) || !(p < 1.f)) return ECHO_ERR_SHAPE;
    if (((uintptr_t)x | (uintptr_t)y | (uintptr_t)mask_bits) & 15u) return ECHO_ERR_ALIGN;
    const size_t n_quads = (n + 3) / 4;
    const float scale = 1.0f / (1.0f - p);
    echo::k_dropout_fwd<<<echo::stream_grid(n_quads), 256, 0, static_cast<hipStream_t>(stream)>>>(
        x, n, p, scale, (uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)offset, (uint32_t)(offset >> 32), y,
        mask_bits, n_quads);
    return hipGetLastError() == hipSuccess ? ECHO_OK : ECHO_ERR_HIP;
}

echo_status_t echo_dropout_bwd(const float *dy, const uint32_t *mask_bits, size_t n, float p, float *dx,
                               void *stream) {
    if (!dy || !dx || !mask_bits) return ECHO_ERR_NULL;
    if (n == 0 || n > echo::kMaxElements || !(p >= 0.f) || !(p < 1.f)) return ECHO_ERR_SHAPE;
    if (((uintptr_t)dy | (uintptr_t)dx | (uintptr_t)mask_bits) & 15u) return ECHO_ERR_ALIGN;
    const size_t n_quads = (n + 3) / 4;
    const float scale = 1.0f / (1.0f - p);
    echo::k_dropout_bwd<<<echo::stream_grid(n_quads), 256, 0, static_cast<hipStream_t>(stream)>>>(
        dy, mask_bits, n, scale, dx, n_quads);
    return hipGetLastError() == hipSuccess ? ECHO_OK : ECHO_ERR_HIP;
}

}  // extern "C"
