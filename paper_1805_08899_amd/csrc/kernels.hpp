// Host-side launch functions of the libechoattn kernels.  Each validates
// nothing (the C ABI layer did) and returns hipGetLastError() after its launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

#include <atomic>

namespace echo {

struct AttnShape {
    int B, Tq, Tk, H, Dv;
    bool bf16;   // Qp, Kp, V, v stored as bf16
    bool acc;    // backward: add into dKp, dV, dv instead of overwriting them (per-step decoder form)
};

// Kernels whose dynamic LDS exceeds the default limit need that limit raised, per device.  `granted` (one table
// per kernel instantiation, zero-initialised) remembers the largest size already granted on each device, so the
// runtime is asked once per device and size instead of on every launch.  Safe to call from several threads: at
// worst two of them ask for the same size.
constexpr int kMaxDevices = 64;
struct LdsGrants { std::atomic<size_t> bytes[kMaxDevices]; };
inline hipError_t ensure_dynamic_lds(const void *kernel, size_t bytes, LdsGrants &granted) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (granted.bytes[dev].load(std::memory_order_acquire) >= bytes) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) granted.bytes[dev].store(bytes, std::memory_order_release);
    return e;
}

// Row pitch (floats) of the dS workspace: keys rounded up to the key tile of
// the recompute kernel, pad entries are written as zeros.
constexpr int kDsPad = 8;
inline int ds_pitch(int Tk) { return (Tk + kDsPad - 1) / kDsPad * kDsPad; }

// F1  scores; tmap != nullptr also writes the tanh map (stash baseline)
hipError_t launch_score(const AttnShape &s, const void *Qp, const void *Kp, const void *v, const int *key_len,
                        float *S, float *tmap, hipStream_t st);
// F1+F2+F3 in one kernel (no workspace); needs H to be a multiple of 4, a row tile that fits LDS and a sample's
// value rows below 2 GiB
bool fwd_fused_supported(const AttnShape &s);
hipError_t launch_fwd_fused(const AttnShape &s, const void *Qp, const void *Kp, const void *V, const void *v,
                            const int *key_len, float *C, float *P, hipStream_t st);
// F2  masked softmax over keys, one wave per (b, i) row
hipError_t launch_softmax(const AttnShape &s, const float *S, const int *key_len, float *P, hipStream_t st);
// F3  context = P . V            (MFMA)
hipError_t launch_context(const AttnShape &s, const float *P, const void *V, const int *key_len, float *C,
                          hipStream_t st);
// B1 + B2 and the sample ranking in one launch:
//   dV = P^T . dC (MFMA);  dP = dC . V^T (MFMA) then dS = P (dP - rowsum(P dP)), dS has row pitch ds_pitch(Tk),
//   ds_rowsum[b*Tq+i] = sum_j dS;
//   order[r] = b | L_b << 16 for the sample with the r-th most valid keys (index order if B > kMaxSortedB)
constexpr int kMaxSortedB = 1024;
// with_ds = false leaves dS and ds_rowsum alone (they are given) and launches only the dV and ranking blocks
hipError_t launch_bwd_pre(const AttnShape &s, const float *dC, const void *V, const float *P, const int *key_len,
                          float *dS, float *ds_rowsum, int *order, float *dV, hipStream_t st, bool with_ds = true);
// B3 + B4  fused recompute: dQp, dKp, per-sample partials of dv (dv_part [B,H]) and, by the blocks that start
// last, dv[h] = sum_b dv_part[b,h] in index order (added to dv if s.acc).  dv_flag: ceil(H/64) x B words of
// workspace in any state; epoch: a number no earlier launch on this workspace used (never 0).
// tmap != nullptr reads tanh from the stashed map instead of recomputing it; dQp == nullptr: dQp is not wanted
hipError_t launch_recompute(const AttnShape &s, const void *Qp, const void *Kp, const void *v, const int *order,
                            const float *dS, const float *ds_rowsum, const float *tmap, float *dQp, float *dKp,
                            float *dv_part, unsigned long long *dv_flag, unsigned long long epoch, float *dv,
                            hipStream_t st);
// B4  dv[h] = sum_b dv_part[b,h], fixed order
hipError_t launch_dv_reduce(const AttnShape &s, const float *dv_part, float *dv, hipStream_t st);
// One decoder step (Tq = 1) of the backward pass in one launch; dKp, dV and dv_part [B,H] are added to.
size_t step_lds_bytes(const AttnShape &s);
hipError_t launch_step_fwd(const AttnShape &s, const void *Qp, const void *Kp, const void *V, const void *v,
                           const int *key_len, float *C, float *P, hipStream_t st);
hipError_t launch_step_bwd(const AttnShape &s, const float *dC, const float *P, const void *Qp, const void *Kp,
                           const void *V, const void *v, const int *key_len, float *dQp, float *dKp, float *dV,
                           float *dv_part, hipStream_t st);

// The same step with the key-side sums deferred: writes dQp [B,1,H], row `step` of every sample's `steps` rows of
// dS (ds_out [B, steps, ds_pitch(Tk)]) and that row's sum (ds_sum_out [B, steps]); reads only.
hipError_t launch_step_bwd_query(const AttnShape &s, const float *dC, const float *P, const void *Qp, const void *Kp,
                                 const void *V, const void *v, const int *key_len, float *dQp, float *ds_out,
                                 float *ds_sum_out, int steps, int step, hipStream_t st);

// Decoder steps on a short key axis (Tk <= 64, H and Dv multiples of 4 up to 512, B <= kStepSplitMaxB) with a
// sample spread over four blocks that exchange one float per key through `mail` (step_split_mail_bytes(s) bytes of
// device memory in any state, used by one launch at a time; 0 bytes: the shape does not qualify).
// step_split_applicable: the shape qualifies and the current device runs all 4 B blocks at once.
// epoch: a number no earlier launch on this mail area used (never 0).
constexpr int kStepSplitMaxB = 64;
size_t step_split_mail_bytes(const AttnShape &s);
bool step_split_applicable(const AttnShape &s);
hipError_t launch_step_fwd_split(const AttnShape &s, const void *Qp, const void *Kp, const void *V, const void *v,
                                 const int *key_len, float *C, float *P, void *mail, unsigned long long epoch,
                                 hipStream_t st);
hipError_t launch_step_bwd_query_split(const AttnShape &s, const float *dC, const float *P, const void *Qp,
                                       const void *Kp, const void *V, const void *v, const int *key_len, float *dQp,
                                       float *ds_out, float *ds_sum_out, int steps, int step, void *mail,
                                       unsigned long long epoch, hipStream_t st);

}  // namespace echo
