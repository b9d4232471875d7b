// Backward pass of one decoder step (Section 2: the decoder produces one query at a time against the same
// encoder states) in ONE launch.  With a single query per sample every quantity of the backward pass except dv
// is local to the sample, so a block takes a sample through all of it:
//   dP[j]  = sum_d dC[d] V[j,d]                      (Eq. 2: from the inputs alone)
//   dS[j]  = P[j] (dP[j] - sum_j P dP)
//   t      = tanh(q[h] + k[j,h]) re-evaluated        (Section 3.4)
//   dQp[h] = v[h] sum_j dS[j] (1 - t^2),   dKp[j,h] += v[h] dS[j] (1 - t^2),   dV[j,:] += P[j] dC
//   dv_part[b,h] += sum_j dS[j] t                    (per sample; summed over the samples once per sentence)
// One launch instead of three.  What bounds a step is memory, not arithmetic: every step reads K and V of the
// valid keys and reads and writes the whole dKp and dV accumulators (23 MB at 64 sentences of 30 keys, H = Dv =
// 512), traffic that the batched call pays once for all steps.  The sum over samples that dv needs is deferred to
// one small launch at the end of the sentence.  Results do not depend on the order in which blocks run: every
// element has one owner.
#include "common.hpp"
#include "kernels.hpp"

namespace echo {

__device__ __forceinline__ float comp4(const float4 &x, int c) { return c == 0 ? x.x : c == 1 ? x.y : c == 2 ? x.z : x.w; }

constexpr int ST_W = 8;                   // waves per block
constexpr int ST_THREADS = 64 * ST_W;
constexpr int ST_KB = 4;                  // keys per wave and batch: a batch of the block is 32 consecutive keys

// Block = (sample b, 64-wide slice of h); it also owns the matching slice of the columns of dV.  Wave w takes
// keys 32 n + 4 w .. + 3 of every batch n; the first batch's K, old dKp and old dV are requested before dP is
// formed.  dP is formed by every h slice of a sample for itself (a few ten thousand multiply-adds, V comes from
// the L2 that the slices of a sample share).
//
// DEFER: the key-side sums are left to one batched call at the end of the sentence.  The step then only reads: it
// writes dQp, and the block of the first h slice writes the step's row of dS (row `ds_row` of the sample's
// `ds_rows` rows of `ds_pitch` floats, zeros at masked keys and pads) and its sum; dKp, dV and dv_part are not
// touched.
template <typename T, bool DEFER>
__global__ __launch_bounds__(ST_THREADS) void k_step_bwd(
    const float *__restrict__ dC, const float *__restrict__ P, const T *__restrict__ Qp, const T *__restrict__ Kp,
    const T *__restrict__ V, const T *__restrict__ v, const int *__restrict__ key_len, float *__restrict__ dQp,
    float *__restrict__ dKp, float *__restrict__ dV, float *__restrict__ dv_part, float *__restrict__ ds_out,
    float *__restrict__ ds_sum_out, int ds_rows, int ds_row, int ds_pitch, int Tk, int H, int Dv, int cw) {
    extern __shared__ float s_step[];     // [Tk] P, then [Tk] dP
    float *s_p = s_step, *s_dp = s_step + Tk;
    __shared__ float s_q[ST_W][64], s_r[ST_W][64];
    const int hs = blockIdx.x, b = blockIdx.y;
    const int lane = lane_id(), w = wave_id();
    const int h = hs * 64 + lane;
    const bool hv = h < H;
    const int hc = hv ? h : H - 1;
    const int L = clamp_len(key_len[b], Tk);
    float *ds_dst = DEFER ? ds_out + ((size_t)b * ds_rows + ds_row) * ds_pitch : nullptr;
    if (DEFER && hs == 0) {               // masked keys and pads of the stored dS row: zeros
        for (int j = L + (int)threadIdx.x; j < ds_pitch; j += ST_THREADS) ds_dst[j] = 0.f;
        if (L == 0 && threadIdx.x == 0) ds_sum_out[(size_t)b * ds_rows + ds_row] = 0.f;
    }
    if (L == 0) {                         // no valid key: the query gets no gradient, the sums get nothing
        if (w == 0 && hv) dQp[(size_t)b * H + h] = 0.f;
        return;
    }
    const float *dCb = dC + (size_t)b * Dv;
    const float *Pb = P + (size_t)b * Tk;
    const T *Vb = V + (size_t)b * Tk * Dv;
    const T *Kb = Kp + (size_t)b * Tk * H;
    float *dKb = dKp + (size_t)b * Tk * H;
    float *dVb = dV + (size_t)b * Tk * Dv;
    const int c_lo = hs * cw, c_hi = min(c_lo + cw, Dv);         // this block's columns of dV
    const int n_batch = (L + 8 * ST_KB - 1) / (8 * ST_KB);

    // ---- requests of the first batch: K and old dKp at this lane's h, old dV at this lane's first column
    float k0[ST_KB], oldk0[ST_KB], oldv0[ST_KB];
    const int c0 = min(c_lo + lane, Dv - 1);
#pragma unroll
    for (int u = 0; u < ST_KB; ++u) {
        const int j = min(ST_KB * w + u, L - 1);
        k0[u] = ld(Kb, (size_t)j * H + hc);
        oldk0[u] = DEFER ? 0.f : dKb[(size_t)j * H + hc];
        oldv0[u] = DEFER ? 0.f : dVb[(size_t)j * Dv + c0];
    }
    const float sq = kTwoLog2e * ld(Qp, (size_t)b * H + hc);
    float v_raw = ld(v, (size_t)hc);     // scaled behind the barrier below: as a guarded load with its scaling it was
                                         // awaited on the spot, before the loads of the dP loop had been requested

    // ---- dP[j] = sum_d dC[d] V[j,d] for this wave's keys of every batch; P to LDS (its first ST_THREADS entries are
    //      requested here and stored behind the loop: stored at once, they were a trip to memory that the loads of the
    //      loop had to wait for)
    const int jp = min((int)threadIdx.x, L - 1);
    const float p_first = Pb[jp];
    for (int n = 0; n < n_batch; ++n) {
        const int j0 = 8 * ST_KB * n + ST_KB * w;
        if (j0 >= L) break;                                       // wave-uniform
        float acc[ST_KB] = {0.f, 0.f, 0.f, 0.f};
        for (int d = 4 * lane; d < Dv; d += 256) {
            const float4 c = ld4(dCb, (size_t)d);
            float4 x[ST_KB];
#pragma unroll
            for (int u = 0; u < ST_KB; ++u) x[u] = ld4(Vb, (size_t)min(j0 + u, L - 1) * Dv + d);
#pragma unroll
            for (int u = 0; u < ST_KB; ++u)
                acc[u] += (c.x * x[u].x + c.y * x[u].y) + (c.z * x[u].z + c.w * x[u].w);
        }
#pragma unroll
        for (int u = 0; u < ST_KB; ++u) {
            const float tot = wave_sum(acc[u]);
            if (lane == 0 && j0 + u < L) s_dp[j0 + u] = tot;
        }
    }
    if ((int)threadIdx.x < L) s_p[threadIdx.x] = p_first;
    for (int j = threadIdx.x + ST_THREADS; j < L; j += ST_THREADS) s_p[j] = Pb[j];
    __syncthreads();
    asm volatile("" : "+v"(v_raw));
    const float v4 = hv ? 4.f * v_raw : 0.f;

    // ---- the two row sums, formed by every wave for itself (same arithmetic, same result in all waves)
    float r = 0.f;
    for (int j = lane; j < L; j += 64) r += s_p[j] * s_dp[j];
    r = wave_sum(r);
    float dsum = 0.f;
    for (int j = lane; j < L; j += 64) dsum += s_p[j] * (s_dp[j] - r);
    dsum = wave_sum(dsum);                // sum_j dS[j]: zero in exact arithmetic; kept so that sum dS t is exact in fp32

    // ---- recomputation at (this wave's keys, this lane's h):  r' = 1 / (exp(2 (q + k)) + 1),
    //      t = 1 - 2 r',  1 - t^2 = 4 r' (1 - r');  and dV at this lane's columns
    float accQ = 0.f, accR = 0.f;
    for (int n = 0; n < n_batch; ++n) {
        const int j0 = 8 * ST_KB * n + ST_KB * w;
        if (j0 >= L) break;                                       // wave-uniform
        float k[ST_KB], oldk[ST_KB];
#pragma unroll
        for (int u = 0; u < ST_KB; ++u) {
            if (n == 0) {
                k[u] = k0[u];
                oldk[u] = oldk0[u];
            } else {
                const size_t at = (size_t)min(j0 + u, L - 1) * H + hc;
                k[u] = ld(Kb, at);
                oldk[u] = DEFER ? 0.f : dKb[at];
            }
        }
#pragma unroll
        for (int u = 0; u < ST_KB; ++u) {
            if (j0 + u < L) {                                     // wave-uniform
                const float ds = s_p[j0 + u] * (s_dp[j0 + u] - r);
                const float rr = fast_rcp(fast_exp2(__builtin_fmaf(kTwoLog2e, k[u], sq)) + 1.0f);
                const float g = ds * __builtin_fmaf(-rr, rr, rr);
                accQ += g;
                accR = __builtin_fmaf(ds, rr, accR);
                if (!DEFER && hv) store_streaming(&dKb[(size_t)(j0 + u) * H + h], __builtin_fmaf(v4, g, oldk[u]));
                if (DEFER && hs == 0 && lane == 0) ds_dst[j0 + u] = ds;
            }
        }
        for (int c = c_lo + lane, m = 0; !DEFER && c < c_hi; c += 64, ++m) {
            const float dc = dCb[c];
#pragma unroll
            for (int u = 0; u < ST_KB; ++u) {
                if (j0 + u < L) {
                    float *at = dVb + (size_t)(j0 + u) * Dv + c;
                    const float old = (n == 0 && m == 0) ? oldv0[u] : *at;
                    store_streaming(at, __builtin_fmaf(s_p[j0 + u], dc, old));
                }
            }
        }
    }
    s_q[w][lane] = accQ;
    s_r[w][lane] = accR;
    __syncthreads();
    if (w == 0 && hv) {
        float tq = 0.f, tr = 0.f;
#pragma unroll
        for (int k2 = 0; k2 < ST_W; ++k2) {
            tq += s_q[k2][lane];
            tr += s_r[k2][lane];
        }
        store_streaming(&dQp[(size_t)b * H + h], v4 * tq);
        if (!DEFER) {
            float *dvp = dv_part + (size_t)b * H + h;
            *dvp += __builtin_fmaf(-2.f, tr, dsum);
        } else if (hs == 0 && lane == 0) {
            ds_sum_out[(size_t)b * ds_rows + ds_row] = dsum;
        }
    }
}

// Forward pass of one decoder step (one query per sample) in one launch of one block per sample: scores with the
// eight waves taking four keys each per batch and the lanes along h, softmax over the valid keys, context with a
// thread per column.  tanh is taken from the exponential of the sum here (one exponential and one reciprocal per
// element): a step is a few thousand elements per wave, nothing to save by factoring it.
template <typename T>
__global__ __launch_bounds__(ST_THREADS) void k_step_fwd(
    const T *__restrict__ Qp, const T *__restrict__ Kp, const T *__restrict__ V, const T *__restrict__ v,
    const int *__restrict__ key_len, float *__restrict__ C, float *__restrict__ P, int Tk, int H, int Dv) {
    extern __shared__ float s_step[];     // [Tk] scores, then probabilities
    float *s_s = s_step;
    const int b = blockIdx.x;
    const int lane = lane_id(), w = wave_id();
    const int L = clamp_len(key_len[b], Tk);
    float *Pb = P + (size_t)b * Tk;
    float *Cb = C + (size_t)b * Dv;
    if (L == 0) {                         // no valid key: zeros
        for (int j = threadIdx.x; j < Tk; j += ST_THREADS) Pb[j] = 0.f;
        for (int d = threadIdx.x; d < Dv; d += ST_THREADS) Cb[d] = 0.f;
        return;
    }
    const T *qb = Qp + (size_t)b * H;
    const T *Kb = Kp + (size_t)b * Tk * H;
    const T *Vb = V + (size_t)b * Tk * Dv;
    const int n_batch = (L + 8 * ST_KB - 1) / (8 * ST_KB);
    const int H4 = (H % 4 == 0) ? H : 0;  // rows are read four elements at a time when every row starts aligned

    // ---- scores: S[j] = sum_h v[h] tanh(q[h] + k[j,h]),  tanh = 1 - 2 / (exp(2 (q + k)) + 1)
    for (int n = 0; n < n_batch; ++n) {
        const int j0 = 8 * ST_KB * n + ST_KB * w;
        float acc[ST_KB] = {0.f, 0.f, 0.f, 0.f};
        if (j0 < L) {                                             // wave-uniform
            for (int h = 4 * lane; h < H4; h += 256) {
                const float4 q4 = ld4(qb, (size_t)h), v4 = ld4(v, (size_t)h);
                float4 k4[ST_KB];
#pragma unroll
                for (int u = 0; u < ST_KB; ++u) k4[u] = ld4(Kb, (size_t)min(j0 + u, L - 1) * H + h);
#pragma unroll
                for (int u = 0; u < ST_KB; ++u) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float x = kTwoLog2e * (comp4(q4, c) + comp4(k4[u], c));
                        acc[u] += comp4(v4, c) * __builtin_fmaf(-2.f, fast_rcp(fast_exp2(x) + 1.0f), 1.0f);
                    }
                }
            }
            for (int h = H4 + lane; h < H; h += 64) {             // rows that do not start aligned: one element at a time
                const float qh = ld(qb, (size_t)h), vh = ld(v, (size_t)h);
#pragma unroll
                for (int u = 0; u < ST_KB; ++u) {
                    const float x = kTwoLog2e * (qh + ld(Kb, (size_t)min(j0 + u, L - 1) * H + h));
                    acc[u] += vh * __builtin_fmaf(-2.f, fast_rcp(fast_exp2(x) + 1.0f), 1.0f);
                }
            }
#pragma unroll
            for (int u = 0; u < ST_KB; ++u) {
                const float tot = wave_sum(acc[u]);
                if (lane == 0 && j0 + u < L) s_s[j0 + u] = tot;
            }
        }
    }
    lds_barrier();

    // ---- softmax over the valid keys: every wave forms the maximum and the sum itself (same arithmetic in all)
    float mx = -INFINITY;
    for (int j = lane; j < L; j += 64) mx = fmaxf(mx, s_s[j]);
    mx = wave_max(mx);
    float z = 0.f;
    for (int j = lane; j < L; j += 64) z += fast_exp2((s_s[j] - mx) * 1.4426950408889634f);
    z = wave_sum(z);
    const float inv = 1.0f / z;
    lds_barrier();
    for (int j = threadIdx.x; j < Tk; j += ST_THREADS) {
        const float p = j < L ? fast_exp2((s_s[j] - mx) * 1.4426950408889634f) * inv : 0.f;
        if (j < L) s_s[j] = p;
        store_streaming(&Pb[j], p);
    }
    lds_barrier();

    // ---- context: a thread per column, eight value rows in flight
    for (int d = threadIdx.x; d < Dv; d += ST_THREADS) {
        float acc = 0.f;
        for (int j0 = 0; j0 < L; j0 += 8) {
            float x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = ld(Vb, (size_t)min(j0 + u, L - 1) * Dv + d);
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (j0 + u < L) acc = __builtin_fmaf(s_s[j0 + u], x[u], acc);
        }
        store_streaming(&Cb[d], acc);
    }
}

// ---------------------------------------------------------------------------------------------------------------
// Short key axes (Tk <= 64, the sentence lengths of Section 2's translation model) with H and Dv up to 512.
// A step on a few dozen keys is a chain of trips to memory, not arithmetic: measured at 64 samples of 50 keys, the
// general kernels spend their time in four dependent rounds of key loads (two batches of keys, two chunks of h)
// after a first trip for key_len, and in waiting for the acknowledgement of the P stores before the value rows are
// used.  Here every load of the step is requested before the first result is awaited -- key rows are clamped with
// Tk, not with the length, so nothing waits for key_len; rows at or beyond the length are loaded and never used
// -- and all stores come last.  Wave w takes keys w, w + 8, ...; with at most 64 keys every wave holds the whole
// score row (one key per lane), so the softmax needs no LDS pass and the context takes its weights by lane reads.
constexpr int SS_KEYS = 64;               // keys a short step covers at most
constexpr int SS_KU = SS_KEYS / ST_W;     // keys per wave
constexpr int SS_CH = 2;                  // chunks of 256 along h
constexpr int SS_MAX_WIDTH = 256 * SS_CH;

template <typename T>
__global__ __launch_bounds__(ST_THREADS) void k_step_fwd_short(
    const T *__restrict__ Qp, const T *__restrict__ Kp, const T *__restrict__ V, const T *__restrict__ v,
    const int *__restrict__ key_len, float *__restrict__ C, float *__restrict__ P, int Tk, int H, int Dv) {
    __shared__ float s_s[SS_KEYS];
    const int b = blockIdx.x;
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane(wave_id());
    const T *qb = Qp + (size_t)b * H;
    const T *Kb = Kp + (size_t)b * Tk * H;
    const T *Vb = V + (size_t)b * Tk * Dv;

    // ---- every request of the step
    const int len_raw = key_len[b];
    float4 q4[SS_CH], v4[SS_CH], k4[SS_CH][SS_KU];
#pragma unroll
    for (int c = 0; c < SS_CH; ++c) {
        if (256 * c < H) {                                        // block-uniform
            const int h = 256 * c + 4 * lane;
            const int hc = min(h, H - 4);
            q4[c] = ld4(qb, (size_t)hc);
            v4[c] = ld4(v, (size_t)hc);
            if (h >= H) v4[c] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int u = 0; u < SS_KU; ++u) k4[c][u] = ld4(Kb, (size_t)min(w + ST_W * u, Tk - 1) * H + hc);
        }
    }
    float vrow[SS_KEYS];                                          // this thread's column of the value rows
    const int d_own = min((int)threadIdx.x, Dv - 1);
#pragma unroll
    for (int j = 0; j < SS_KEYS; ++j)
        if (j < Tk) vrow[j] = ld(Vb, (size_t)j * Dv + d_own);
    const int L = clamp_len(len_raw, Tk);

    // ---- scores: S[j] = sum_h v[h] tanh(q[h] + k[j,h]),  tanh = 1 - 2 / (exp(2 (q + k)) + 1)
#pragma unroll
    for (int u = 0; u < SS_KU; ++u) {
        const int j = w + ST_W * u;
        if (j < L) {                                              // wave-uniform
            float acc = 0.f;
#pragma unroll
            for (int c = 0; c < SS_CH; ++c) {
                if (256 * c < H) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float x = kTwoLog2e * (comp4(q4[c], e) + comp4(k4[c][u], e));
                        acc += comp4(v4[c], e) * __builtin_fmaf(-2.f, fast_rcp(fast_exp2(x) + 1.0f), 1.0f);
                    }
                }
            }
            const float tot = wave_sum(acc);
            if (lane == 0) s_s[j] = tot;
        }
    }
    lds_barrier();

    // ---- softmax over the valid keys, one key per lane, the same in every wave
    const float sc = lane < L ? s_s[lane] : -INFINITY;
    const float mx = wave_max(sc);
    const float ex = lane < L ? fast_exp2((sc - mx) * 1.4426950408889634f) : 0.f;
    const float z = wave_sum(ex);
    const float p = lane < L ? ex * (1.0f / z) : 0.f;

    // ---- context: a thread per column, the value rows are in registers
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < SS_KEYS; ++j)
        if (j < L) acc = __builtin_fmaf(lane_value(p, j), vrow[j], acc);
    if ((int)threadIdx.x < Dv) store_streaming(&C[(size_t)b * Dv + threadIdx.x], acc);
    if (w == 0 && lane < Tk) store_streaming(&P[(size_t)b * Tk + lane], p);
}

static bool step_fwd_short_ok(const AttnShape &s) {
    return s.Tk <= SS_KEYS && s.H % 4 == 0 && s.H >= 4 && s.H <= SS_MAX_WIDTH && s.Dv <= ST_THREADS;
}

hipError_t launch_step_fwd(const AttnShape &s, const void *Qp, const void *Kp, const void *V, const void *v,
                           const int *key_len, float *C, float *P, hipStream_t st) {
    if (step_fwd_short_ok(s)) {
        if (s.bf16)
            k_step_fwd_short<bf16_t><<<s.B, ST_THREADS, 0, st>>>((const bf16_t *)Qp, (const bf16_t *)Kp,
                                                                 (const bf16_t *)V, (const bf16_t *)v, key_len, C, P,
                                                                 s.Tk, s.H, s.Dv);
        else
            k_step_fwd_short<float><<<s.B, ST_THREADS, 0, st>>>((const float *)Qp, (const float *)Kp, (const float *)V,
                                                                (const float *)v, key_len, C, P, s.Tk, s.H, s.Dv);
        return hipGetLastError();
    }
    const size_t lds = (size_t)s.Tk * sizeof(float);
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    if (lds > 48 * 1024) {
        static LdsGrants granted_bf16, granted_f32;
        hipError_t e = s.bf16 ? ensure_dynamic_lds((const void *)k_step_fwd<bf16_t>, lds, granted_bf16)
                              : ensure_dynamic_lds((const void *)k_step_fwd<float>, lds, granted_f32);
        if (e != hipSuccess) return e;
    }
    if (s.bf16)
        k_step_fwd<bf16_t><<<s.B, ST_THREADS, lds, st>>>((const bf16_t *)Qp, (const bf16_t *)Kp, (const bf16_t *)V,
                                                         (const bf16_t *)v, key_len, C, P, s.Tk, s.H, s.Dv);
    else
        k_step_fwd<float><<<s.B, ST_THREADS, lds, st>>>((const float *)Qp, (const float *)Kp, (const float *)V,
                                                        (const float *)v, key_len, C, P, s.Tk, s.H, s.Dv);
    return hipGetLastError();
}

size_t step_lds_bytes(const AttnShape &s) { return 2 * (size_t)s.Tk * sizeof(float); }

template <typename T, bool DEFER>
static hipError_t launch_step_bwd_t(const AttnShape &s, const float *dC, const float *P, const void *Qp,
                                    const void *Kp, const void *V, const void *v, const int *key_len, float *dQp,
                                    float *dKp, float *dV, float *dv_part, float *ds_out, float *ds_sum_out,
                                    int ds_rows, int ds_row, hipStream_t st) {
    const size_t lds = step_lds_bytes(s);
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    if (lds > 40 * 1024) {
        static LdsGrants granted;
        hipError_t e = ensure_dynamic_lds((const void *)k_step_bwd<T, DEFER>, lds, granted);
        if (e != hipSuccess) return e;
    }
    const int n_hs = (s.H + 63) / 64;
    const int cw = (s.Dv + n_hs - 1) / n_hs;                     // columns of dV per h slice
    dim3 grid(n_hs, s.B);
    k_step_bwd<T, DEFER><<<grid, ST_THREADS, lds, st>>>(dC, P, (const T *)Qp, (const T *)Kp, (const T *)V,
                                                        (const T *)v, key_len, dQp, dKp, dV, dv_part, ds_out,
                                                        ds_sum_out, ds_rows, ds_row, ds_pitch(s.Tk), s.Tk, s.H, s.Dv,
                                                        cw);
    return hipGetLastError();
}

hipError_t launch_step_bwd(const AttnShape &s, const float *dC, const float *P, const void *Qp, const void *Kp,
                           const void *V, const void *v, const int *key_len, float *dQp, float *dKp, float *dV,
                           float *dv_part, hipStream_t st) {
    return s.bf16 ? launch_step_bwd_t<bf16_t, false>(s, dC, P, Qp, Kp, V, v, key_len, dQp, dKp, dV, dv_part, nullptr,
                                                     nullptr, 1, 0, st)
                  : launch_step_bwd_t<float, false>(s, dC, P, Qp, Kp, V, v, key_len, dQp, dKp, dV, dv_part, nullptr,
                                                    nullptr, 1, 0, st);
}

hipError_t launch_step_bwd_query(const AttnShape &s, const float *dC, const float *P, const void *Qp, const void *Kp,
                                 const void *V, const void *v, const int *key_len, float *dQp, float *ds_out,
                                 float *ds_sum_out, int steps, int step, hipStream_t st) {
    return s.bf16 ? launch_step_bwd_t<bf16_t, true>(s, dC, P, Qp, Kp, V, v, key_len, dQp, nullptr, nullptr, nullptr,
                                                    ds_out, ds_sum_out, steps, step, st)
                  : launch_step_bwd_t<float, true>(s, dC, P, Qp, Kp, V, v, key_len, dQp, nullptr, nullptr, nullptr,
                                                   ds_out, ds_sum_out, steps, step, st);
}

}  // namespace echo
