/*
 * The non-linear block of an LSTM cell with its activations recomputed in the backward pass, for MI355X
 * (gfx950); part of libechoattn.so.
 *
 * The Echo paper (Section 2, the LSTM cell) describes the block as slicing and element-wise operations that
 * take the two fully-connected outputs Gx, Gh (each [B, 4H]) and the previous cell state ([B, H]) to the new
 * hidden and cell state, and names the feature maps of the RNN layers as the second target of recomputation
 * (abstract, Section 3.2).  It prints no formula for the block; the textbook cell is used, gates sliced in the
 * order input, forget, candidate, output:
 *
 *   a = Gx + Gh
 *   i = sigmoid(a[:, 0:H])   f = sigmoid(a[:, H:2H])   g = tanh(a[:, 2H:3H])   o = sigmoid(a[:, 3H:4H])
 *   c = f * c_prev + i * g            h = o * tanh(c)
 *
 *   tc = tanh(c)   do = dh * tc   dct = dc + dh * o * (1 - tc^2)   dc_prev = dct * f
 *   da = [dct * g * i (1 - i),  dct * c_prev * f (1 - f),  dct * i * (1 - g^2),  do * o (1 - o)]
 *
 * Recompute path: the forward pass keeps only a, the single sum (Section 4.1: keeping the sum takes half of
 * what keeping both addends would), and the backward pass re-evaluates i, f, g, o, c and tanh(c) from a and
 * c_prev in registers.  Stash path (comparison only): the forward pass writes the four activations and
 * tanh(c), the backward pass reads them.
 *
 * Conventions: all tensors are caller-owned DEVICE memory, fp32, row-major and contiguous, 16-byte aligned.
 * B >= 1, H >= 1 (rows are processed four elements at a time when H is a multiple of 4, one at a time
 * otherwise).  `a` may be the very buffer passed as Gx or as Gh (every element is read before it is written,
 * by the same lane); no other overlap between inputs and outputs is allowed.  dc may be NULL: no gradient
 * reaches c from a later step.  da is the gradient of Gx and of Gh alike.  Outputs are overwritten.  Work is
 * enqueued on `stream` (hipStream_t as void*); no synchronisation, no allocation, no global state.
 * Errors: ECHO_ERR_NULL, ECHO_ERR_SHAPE (B or H < 1, or B * H beyond 2^38), ECHO_ERR_ALIGN, ECHO_ERR_HIP.
 */
#ifndef ECHOLSTM_H
#define ECHOLSTM_H

#include <stddef.h>
#include <stdint.h>

#include "echoattn.h" /* echo_status_t */

#ifdef __cplusplus
extern "C" {
#endif

/* Forward of the block (Section 2, LSTM cell): h [B, H], c [B, H] and the kept sum a [B, 4H]. */
echo_status_t echo_lstm_cell_fwd(int64_t B, int64_t H, const float *Gx, const float *Gh, const float *c_prev,
                                 float *h, float *c, float *a, void *stream);

/* Backward with the activations recomputed from a and c_prev (Section 3.4: redo the forward computation when
 * the backward pass starts): da [B, 4H], dc_prev [B, H]. */
echo_status_t echo_lstm_cell_bwd(int64_t B, int64_t H, const float *dh, const float *dc, const float *a,
                                 const float *c_prev, float *da, float *dc_prev, void *stream);

/* Comparison only (Section 4.1, the baseline keeps the outputs of the operators): the forward pass also
 * writes acts [B, 4H] = (i, f, g, o) and tanh_c [B, H] and keeps no sum; the backward pass reads them. */
echo_status_t echo_lstm_cell_fwd_stash(int64_t B, int64_t H, const float *Gx, const float *Gh,
                                       const float *c_prev, float *h, float *c, float *acts, float *tanh_c,
                                       void *stream);
echo_status_t echo_lstm_cell_bwd_stash(int64_t B, int64_t H, const float *dh, const float *dc,
                                       const float *acts, const float *tanh_c, const float *c_prev, float *da,
                                       float *dc_prev, void *stream);

/* Bytes kept between the forward and the backward pass of one cell, c_prev included:
 * recompute 5 * B * H * 4, stash 6 * B * H * 4. */
size_t echo_lstm_cell_kept_bytes(int64_t B, int64_t H, int stash);

#ifdef __cplusplus
}
#endif
#endif /* ECHOLSTM_H */
