/*
 * libechoattn -- additive (MLP) attention for MI355X (gfx950), forward and
 * backward, with the B x Tq x Tk x H tanh feature map recomputed in the
 * backward pass instead of stashed.
 *
 * The layer (Echo paper, Section 2, attention steps 1 and 2; Section 4.1, the
 * broadcast add + tanh scoring function; Section 5.1, what replaces the T^2 x N
 * feature map):
 *
 *   L_b        = clamp(key_len[b], 0, Tk)
 *   S[b,i,j]   = sum_h v[h] * tanh(Qp[b,i,h] + Kp[b,j,h])            j <  L_b
 *   P[b,i,j]   = softmax over j < L_b of S[b,i,:];   exactly 0.0 for j >= L_b
 *   C[b,i,d]   = sum_j P[b,i,j] * V[b,j,d]
 *
 * Backward from dC (Section 3.2: tanh' = 1 - tanh^2; Eq. 2: gradients of the
 * dense contractions need only their inputs; Section 3.4: the cheap nodes are
 * re-run when the backward pass starts):
 *
 *   dV[b,j,d]  = sum_i P[b,i,j] * dC[b,i,d]
 *   dP[b,i,j]  = sum_d dC[b,i,d] * V[b,j,d]
 *   dS[b,i,j]  = P[b,i,j] * (dP[b,i,j] - sum_j' P[b,i,j'] dP[b,i,j'])
 *   t          = tanh(Qp[b,i,h] + Kp[b,j,h])                (recomputed)
 *   dQp[b,i,h] = sum_j dS[b,i,j] v[h] (1 - t^2)
 *   dKp[b,j,h] = sum_i dS[b,i,j] v[h] (1 - t^2)
 *   dv[h]      = sum_{b,i,j} dS[b,i,j] t
 *
 * Conventions common to every call
 *   - All tensors are row-major, contiguous, innermost index last.
 *   - Every pointer except the descriptor is DEVICE memory owned by the caller
 *     and must be 16-byte aligned.  The library never allocates, frees or
 *     keeps a pointer.
 *   - Qp, Kp, V, v have the element type desc->in_dtype (fp32, or bf16 stored
 *     as 16-bit patterns); all arithmetic and every output is fp32.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) and the call returns without synchronising.  The return
 *     value reports argument validation and launch errors only.
 *   - Outputs are overwritten, never accumulated into.  Rows of P, dKp and dV
 *     at masked keys (j >= L_b) are written as exact zeros.  A sample with
 *     L_b == 0 yields zeros in all of its outputs and adds nothing to dv.
 *   - key_len values are clamped, not validated (that would need a sync).
 *   - Results are bit-identical from run to run: no floating-point atomics.
 *   - Calls are re-entrant; calls that share a workspace must be ordered by
 *     the caller (same stream, or events).  What the library keeps between calls is per host thread and
 *     never affects results: the text of the thread's last error (echo_last_error_detail), the event records
 *     of echo_attn_profile_* while profiling is enabled on that thread, a process-wide counter that numbers
 *     backward launches, and a note per device of kernels whose on-chip memory limit has been raised.
 *   - A HIP error left pending on the calling thread by earlier, unrelated HIP calls is cleared when a call
 *     launches a kernel, so that ECHO_ERR_HIP always refers to the library's own launch.
 */
#ifndef ECHOATTN_H
#define ECHOATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ECHO_OK = 0,
    ECHO_ERR_NULL = 1,       /* a required pointer is NULL */
    ECHO_ERR_SHAPE = 2,      /* a shape outside what the library takes, see "Shape limits" below */
    ECHO_ERR_DTYPE = 3,      /* in_dtype is not one of echo_dtype_t */
    ECHO_ERR_WORKSPACE = 4,  /* workspace_bytes smaller than the matching *_workspace_bytes() */
    ECHO_ERR_ALIGN = 5,      /* a device pointer is not 16-byte aligned */
    ECHO_ERR_HIP = 6         /* a kernel launch failed (hipGetLastError) */
} echo_status_t;

typedef enum { ECHO_F32 = 0, ECHO_BF16 = 1 } echo_dtype_t; /* storage of Qp, Kp, V, v */

/* Shape limits.  Every call returns ECHO_ERR_SHAPE, before anything is launched, unless
 *   - B, Tq, Tk, H, Dv are all >= 1;
 *   - Dv is a multiple of 4 (value rows are read 16 bytes at a time);
 *   - Tk <= ECHO_ATTN_MAX_TK (16 rows of dP over all keys sit in on-chip memory in the softmax backward);
 *     the echo_attn_step_* calls take Tk <= ECHO_ATTN_STEP_MAX_TK instead;
 *   - B <= ECHO_ATTN_MAX_B (the batch is one dimension of the launch grid);
 *   - each per-sample tensor (Tq*H, Tk*H, Tk*Dv, Tq*Dv, Tq*(Tk+16) elements) stays below 2^31 elements and
 *     B*Tq*Tk*H below 2^62;
 *   - for the echo_attn_step_* calls, Tq == 1.
 * H may be any value >= 1: shapes whose H is not a multiple of 4, or whose tile of query rows does not fit
 * on-chip memory (H above about 4600), run through separate score / softmax / context kernels. */
#define ECHO_ATTN_MAX_TK 2048
#define ECHO_ATTN_STEP_MAX_TK 8192
#define ECHO_ATTN_MAX_B 65535

typedef struct {
    int32_t B;        /* batch                      */
    int32_t Tq;       /* queries per sample         */
    int32_t Tk;       /* keys per sample            */
    int32_t H;        /* attention hidden size      */
    int32_t Dv;       /* value width                */
    int32_t in_dtype; /* echo_dtype_t               */
} echo_attn_desc_t;

/* Scratch the two passes need, in bytes (host arithmetic; 0 on an invalid
 * descriptor).  Workspace contents need not survive between calls and may start in any state: the only
 * state that persists from forward to backward is P (Section 5.1).
 * The forward pass needs none (0 is returned, and echo_attn_fwd then accepts workspace == NULL) whenever its
 * one-kernel form runs, which keeps the scores on chip: H a multiple of 4, a tile of eight query rows
 * within on-chip memory and a sample's V below 2 GiB, i.e. every shape of practical size; otherwise B*Tq*Tk
 * floats for the scores.
 * Exception, decoder steps: for Tq == 1, Tk <= 64, H and Dv multiples of 4 up to 512 and B <= 64 the forward call
 * asks for 4 KB per sample, through which the four blocks that share a sample pass the scores to one another (see
 * echo_attn_fwd). */
size_t echo_attn_fwd_workspace_bytes(const echo_attn_desc_t *desc);
size_t echo_attn_bwd_workspace_bytes(const echo_attn_desc_t *desc);

/* Forward (Section 2, steps 1-2; scoring function of Section 4.1).
 *   in : Qp [B,Tq,H], Kp [B,Tk,H], V [B,Tk,Dv], v [H]   (in_dtype), key_len [B] int32
 *   out: context [B,Tq,Dv] fp32, P [B,Tq,Tk] fp32 (keep it for the backward call)
 * The tanh map is never written to memory.
 * Tq == 1 is a decoder step (Section 2: one query per sample against the same encoder states) and runs the
 * kernels made for it.  On a short key axis (the shapes listed at echo_attn_fwd_workspace_bytes) a sample is
 * spread over four blocks that wait for one another's scores, bounded by 2 s: if the GPU is so occupied by other
 * work that the four do not get to run together within that time, context and P of the call are NaN.  The
 * workspace then carries the scores between them: one call at a time per workspace, also across streams. */
echo_status_t echo_attn_fwd(const echo_attn_desc_t *desc,
                            const void *Qp, const void *Kp, const void *V, const void *v,
                            const int32_t *key_len,
                            float *context, float *P,
                            void *workspace, size_t workspace_bytes, void *stream);

/* Backward (Section 3.4 recomputation fused into one kernel as in the
 * hand-tuned variant of Section 6.1; Section 3.2 and Eq. 2 for the rules).
 *   in : dContext [B,Tq,Dv] fp32, P [B,Tq,Tk] fp32 as written by echo_attn_fwd,
 *        and the forward inputs
 *   out: dQp [B,Tq,H], dKp [B,Tk,H], dV [B,Tk,Dv], dv [H], all fp32 */
echo_status_t echo_attn_bwd(const echo_attn_desc_t *desc,
                            const float *dContext, const float *P,
                            const void *Qp, const void *Kp, const void *V, const void *v,
                            const int32_t *key_len,
                            float *dQp, float *dKp, float *dV, float *dv,
                            void *workspace, size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory or hand over a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): echo_attn_bwd with the workspace taken from a buffer of
 * ECHO_ATTN_STATIC_SCRATCH_BYTES that is part of the library's device image (every GPU the library runs on holds
 * one until the process ends).  Same arguments, kernels and results as echo_attn_bwd; calls no allocator.
 *   - The device that `stream` belongs to must be the current device of the calling thread.  The first call on
 *     a device looks up the address of that device's buffer (no allocation); later calls reuse it.
 *   - ECHO_ERR_WORKSPACE if echo_attn_bwd_workspace_bytes(desc) exceeds ECHO_ATTN_STATIC_SCRATCH_BYTES
 *     (echo_last_error_detail() then names both sizes); nothing is launched.
 *   - All calls on one GPU share that GPU's buffer, which keeps the last call's contents (nothing in it has to
 *     be cleared between calls): two calls that may overlap on one GPU (different streams without an event
 *     between them, several host threads) race, and so does a graph replayed concurrently with itself. */
#define ECHO_ATTN_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
echo_status_t echo_attn_bwd_static(const echo_attn_desc_t *desc,
                                   const float *dContext, const float *P,
                                   const void *Qp, const void *Kp, const void *V, const void *v,
                                   const int32_t *key_len,
                                   float *dQp, float *dKp, float *dV, float *dv,
                                   void *stream);

/* Backward of one decoder step (Section 2: the decoder produces one query at a time against the same encoder
 * states, so Kp, V and v are shared by all steps of a sentence and their gradients are sums over the steps).
 * Same as echo_attn_bwd, except that dKp, dV and dv are ADDED TO instead of overwritten: the caller clears them
 * before the first step (rows at masked keys then stay exact zeros) and calls this once per step, with that
 * step's Qp [B,Tq,H], P and dContext (Tq is usually 1), in any order.  dQp [B,Tq,H] is overwritten.
 * The result after all steps equals echo_attn_bwd on the steps stacked along Tq, up to the order of additions. */
echo_status_t echo_attn_bwd_accumulate(const echo_attn_desc_t *desc,
                                       const float *dContext, const float *P,
                                       const void *Qp, const void *Kp, const void *V, const void *v,
                                       const int32_t *key_len,
                                       float *dQp, float *dKp, float *dV, float *dv,
                                       void *workspace, size_t workspace_bytes, void *stream);

/* The same decoder step in one launch per direction (Tq must be 1; Tk <= ECHO_ATTN_STEP_MAX_TK; no workspace).
 * echo_attn_step_fwd: same results as echo_attn_fwd with Tq = 1 (context [B,1,Dv] and P [B,1,Tk] overwritten).
 * echo_attn_step_bwd: with one query per sample everything but dv
 * is local to a sample, so one kernel takes each sample through dP, the softmax backward, the recomputation of
 * tanh (Section 3.4) and dV; no workspace.  dQp [B,1,H] is overwritten; dKp [B,Tk,H], dV [B,Tk,Dv] and
 * dv_part [B,H] (per-sample parts of dv) are ADDED TO: the caller clears them before the first step of a
 * sentence.  After the last step echo_attn_step_finish adds the per-sample parts in index order:
 * dv[h] = sum_b dv_part[b,h] (dv is overwritten).  Results equal echo_attn_bwd on the steps stacked along Tq up
 * to the order of additions, and are reproducible for a given order of calls.
 * Errors as echo_attn_bwd; ECHO_ERR_SHAPE also for Tq != 1; the key axis may be as long as
 * ECHO_ATTN_STEP_MAX_TK. */
echo_status_t echo_attn_step_fwd(const echo_attn_desc_t *desc,
                                 const void *Qp, const void *Kp, const void *V, const void *v,
                                 const int32_t *key_len, float *context, float *P, void *stream);
echo_status_t echo_attn_step_bwd(const echo_attn_desc_t *desc,
                                 const float *dContext, const float *P,
                                 const void *Qp, const void *Kp, const void *V, const void *v,
                                 const int32_t *key_len,
                                 float *dQp, float *dKp, float *dV, float *dv_part, void *stream);
echo_status_t echo_attn_step_finish(const echo_attn_desc_t *desc, const float *dv_part, float *dv, void *stream);

/* Decoder steps with the key-side gradients left to the end of the sentence.  Only dQp of step t is needed before
 * step t - 1 can run (Section 2: the query of a step comes from the decoder state of that step); dKp, dV and dv
 * are sums over all steps (Kp, V and v are shared by them), so nothing forces the steps to add to them one by
 * one: that costs a read and a write of all of dKp and dV per step.  Instead
 *   echo_attn_step_bwd_query   (once per step, any order) forms that step's dP and dS (Eq. 2, softmax backward),
 *       re-evaluates tanh (Section 3.4) and writes dQp [B,1,H]; it also leaves the step's row of dS and its sum in
 *       `ds_rows`, a device buffer of echo_attn_steps_ds_bytes(sentence descriptor) bytes that the caller keeps
 *       for the sentence (any initial state).  It reads Kp and V once and writes nothing else.  `desc` has
 *       Tq == 1; `step` in [0, steps) is the position of this step in the stacked tensors below.  On a short key
 *       axis it spreads a sample over four blocks as echo_attn_fwd does with Tq == 1 (same shapes, same bounded
 *       wait, dQp and the step's row NaN if it runs out); `ds_rows` carries what they exchange, so the step calls
 *       of one `ds_rows` must not overlap one another.
 *   echo_attn_steps_bwd_keys   (once per sentence, after all steps) forms dKp [B,Tk,H], dV [B,Tk,Dv] and dv [H]
 *       (overwritten) from the steps stacked along Tq: dContext [B,steps,Dv], P [B,steps,Tk], Qp [B,steps,H], and
 *       `ds_rows` as the steps left it.  `desc` has Tq == steps.  Workspace: echo_attn_bwd_workspace_bytes(desc).
 * Results equal echo_attn_bwd on the stacked steps up to the order of additions and are reproducible.
 * Errors as echo_attn_bwd; ECHO_ERR_SHAPE also for Tq != 1 in the step call or step outside [0, steps). */
size_t echo_attn_steps_ds_bytes(const echo_attn_desc_t *sentence_desc);
echo_status_t echo_attn_step_bwd_query(const echo_attn_desc_t *desc, int32_t step, int32_t steps,
                                       const float *dContext, const float *P,
                                       const void *Qp, const void *Kp, const void *V, const void *v,
                                       const int32_t *key_len,
                                       float *dQp, void *ds_rows, void *stream);
echo_status_t echo_attn_steps_bwd_keys(const echo_attn_desc_t *desc,
                                       const float *dContext, const float *P,
                                       const void *Qp, const void *Kp, const void *v,
                                       const int32_t *key_len, const void *ds_rows,
                                       float *dKp, float *dV, float *dv,
                                       void *workspace, size_t workspace_bytes, void *stream);

/* Comparison only: the baseline behaviour of Section 4.1, which stashes the
 * output of tanh as a feature map.  Same results as the pair above;
 * `tanh_map` is B*Tq*Tk*H fp32 (echo_attn_stash_bytes), written by the
 * forward call and read by the backward call in place of the recomputation. */
size_t echo_attn_stash_bytes(const echo_attn_desc_t *desc);
size_t echo_attn_fwd_stash_workspace_bytes(const echo_attn_desc_t *desc);   /* workspace of echo_attn_fwd_stash */
echo_status_t echo_attn_fwd_stash(const echo_attn_desc_t *desc,
                                  const void *Qp, const void *Kp, const void *V, const void *v,
                                  const int32_t *key_len,
                                  float *context, float *P, float *tanh_map,
                                  void *workspace, size_t workspace_bytes, void *stream);
echo_status_t echo_attn_bwd_stash(const echo_attn_desc_t *desc,
                                  const float *dContext, const float *P, const float *tanh_map,
                                  const void *V, const void *v,
                                  const int32_t *key_len,
                                  float *dQp, float *dKp, float *dV, float *dv,
                                  void *workspace, size_t workspace_bytes, void *stream);

/* Per-kernel timing for the benchmark.  While enabled, every kernel the
 * library launches from the calling thread is bracketed by HIP events on its
 * stream.  echo_attn_profile_read() synchronises those events and copies up
 * to `cap` entries (kernel name, launches, total milliseconds) to HOST arrays,
 * returns the number of distinct kernels, and clears the record.  Enabling
 * costs two event records per launch; leave it off otherwise. */
void echo_attn_profile_enable(int on);
int  echo_attn_profile_read(const char **names, int *launches, float *total_ms, int cap);

/* Measurement support: launches one synthetic kernel on `stream` so that the
 * caller can time the machine's ceilings with its own events.
 *   ECHO_CAL_FMA / RCP / EXP2   every lane issues nothing but v_fma_f32 /
 *                               v_rcp_f32 / v_exp_f32 in 16 independent chains
 *   ECHO_CAL_FWD_MIX            the per-tanh instruction mix of the score loop
 *                               (fma, rcp, fma); *work counts tanh evaluations
 *   ECHO_CAL_BWD_MIX            the mix of the recompute loop (fma, rcp, 4 fma)
 *   ECHO_CAL_COPY               dst[i] = src[i] over `bytes` bytes (16-byte units)
 * ALU kinds launch `blocks` blocks of 256 lanes, each running `iters` loop
 * trips, and write one float per lane to dst (bytes >= blocks*256*4).
 * *work (HOST) receives the number of lane-instructions (FMA/RCP/EXP2), of
 * tanh-equivalents (mixes) or of bytes copied (COPY; read + write is twice that). */
typedef enum { ECHO_CAL_FMA = 0, ECHO_CAL_RCP = 1, ECHO_CAL_EXP2 = 2, ECHO_CAL_FWD_MIX = 3,
               ECHO_CAL_BWD_MIX = 4, ECHO_CAL_COPY = 5 } echo_cal_kind_t;
echo_status_t echo_attn_calibrate(int kind, int blocks, int iters, const void *src, void *dst, size_t bytes,
                                  double *work, void *stream);

const char *echo_status_string(echo_status_t s);
/* Kernel name and HIP error text of the calling thread's last ECHO_ERR_HIP, or the two sizes of
 * echo_attn_bwd_static's last ECHO_ERR_WORKSPACE ("" if none). */
const char *echo_last_error_detail(void);
const char *echo_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ECHOATTN_H */
