/*
 * Dropout whose feature map is one bit per element, for MI355X (gfx950); part of libechoattn.so.
 *
 * The Echo paper (Section 5.2) encodes the feature maps of dropout layers to 1 bit in the forward pass and
 * decodes them back to 32 bits in the backward pass.  With inverted dropout
 *
 *   keep_i = (u_i >= p)                     u_i uniform in [0, 1)
 *   y_i    = keep_i ? x_i / (1 - p) : 0
 *   dx_i   = keep_i ? dy_i / (1 - p) : 0
 *
 * the only thing the backward pass needs is keep_i: bit (i mod 32) of 32-bit word (i div 32) of `mask_bits`,
 * 1/32 of the fp32 mask (or of y) that would be kept otherwise.
 *
 * Random numbers: Philox4x32-10 (Salmon et al., SC 2011), a counter-based generator, so that a caller (or a
 * checker) can reproduce them: element i takes output word (i mod 4) of the block with counter
 * (lo32(i div 4), hi32(i div 4), lo32(offset), hi32(offset)) and key (lo32(seed), hi32(seed));
 * u = (word >> 8) * 2^-24, compared with p in fp32.  Use a new `offset` (or seed) for every call that must
 * draw fresh numbers.
 *
 * Conventions: x, y, dy, dx, mask_bits are caller-owned DEVICE memory, 16-byte aligned; n elements, any n >= 1;
 * mask_bits holds echo_dropout_mask_words(n) words, the padding bits of the last word are written as zeros.
 * 0 <= p < 1.  Work is enqueued on `stream` (hipStream_t as void*), no synchronisation, no allocation.
 * Inputs and outputs must not overlap.
 */
#ifndef ECHODROPOUT_H
#define ECHODROPOUT_H

#include <stddef.h>
#include <stdint.h>

#include "echoattn.h" /* echo_status_t */

#ifdef __cplusplus
extern "C" {
#endif

/* Words of the one-bit feature map of n elements: ceil(n / 32). */
size_t echo_dropout_mask_words(size_t n);

/* Forward: y and the one-bit feature map (Section 5.2, encode).
 * Errors: ECHO_ERR_NULL, ECHO_ERR_SHAPE (n == 0, n beyond 2^40 or p outside [0, 1)), ECHO_ERR_ALIGN, ECHO_ERR_HIP. */
echo_status_t echo_dropout_fwd(const float *x, size_t n, float p, uint64_t seed, uint64_t offset,
                               float *y, uint32_t *mask_bits, void *stream);

/* Backward from the one-bit feature map (Section 5.2, decode). */
echo_status_t echo_dropout_bwd(const float *dy, const uint32_t *mask_bits, size_t n, float p,
                               float *dx, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ECHODROPOUT_H */
