// Decoder steps (Section 2: one query per sample against the same encoder states) on a short key axis, with every
// sample spread over FOUR blocks.
//
// A step over a few dozen keys moves 200 KB per sample (the key rows and the value rows) and does next to no
// arithmetic.  With one block per sample a batch of 64 sentences keeps 64 of the 256 compute units busy, and one
// compute unit draws its 200 KB at a small fraction of what the memory system delivers to the whole chip: the
// per-sample kernels measure 7 to 9 us of which the loads are most.  Here a sample is spread over four blocks,
// each of which loads a quarter of the rows that feed the sum over all keys, and a quarter of the columns that
// come after it:
//   forward   part p:  scores of the keys j = p, p + 4, ..   ->  exchange  ->  softmax  ->  context columns of part p
//   backward  part p:  dP of the keys j = p, p + 4, ..       ->  exchange  ->  dS       ->  dQp at the h of part p
// The exchange is one float per key and goes through device memory that the caller provides (a "mail" area of
// step_split_mail_bytes): every part writes its values into one box per receiving part and then takes the other
// parts' values from its own boxes.  A box slot is two 64-bit words, each holding the value next to one half of
// the launch's 64-bit number; a slot is taken once both halves and both copies of the value agree, so the area may
// start in any state, no ordering between stores is needed, and the receiver -- the only reader of its boxes --
// sets them back to zero, so that a captured launch (whose number is fixed at capture) can be replayed.  The four
// blocks of a sample wait for one another, so all of them must be running at once: the launcher uses this form
// only while 4 B blocks fit the compute units of the device, and every wait is bounded (the step's outputs are
// NaN if a value never arrives).
#include "common.hpp"
#include "kernels.hpp"

namespace echo {

constexpr int SP_PARTS = 4;                   // blocks per sample
constexpr int SP_W = 8;                       // waves per block
constexpr int SP_THREADS = 64 * SP_W;
constexpr int SP_KEYS = 64;                   // longest key axis
constexpr int SP_KU = SP_KEYS / SP_PARTS / SP_W;   // keys per wave before the exchange (2): key p + 4 (w + 8 u)
constexpr int SP_CH = 2;                      // 256-wide chunks of the axis that is summed before the exchange
constexpr int SP_COLS = 128;                  // columns (h) per part after the exchange: ceil(width / 4) <= 128
constexpr int SP_GROUPS = SP_THREADS / SP_COLS;    // row groups per block after the exchange (4): key g + 4 m
constexpr int SP_ROWS = SP_KEYS / SP_GROUPS;  // rows per thread (16)
constexpr int SP_MAX_WIDTH = 256 * SP_CH;     // H and Dv up to 512
constexpr unsigned long long kMailSalt = 0x9E3779B9ull;

struct alignas(16) MailSlot {
    unsigned long long w0, w1;
};

__device__ __forceinline__ float comp4s(const float4 &x, int c) { return c == 0 ? x.x : c == 1 ? x.y : c == 2 ? x.z : x.w; }

__device__ __forceinline__ void mail_put(MailSlot *s, float x, unsigned long long epoch) {
    const unsigned long long bits = __float_as_uint(x);
    store_agent(&s->w0, ((epoch & 0xffffffffull) << 32) | bits);
    store_agent(&s->w1, ((((epoch >> 32) ^ kMailSalt) & 0xffffffffull) << 32) | bits);
}
__device__ __forceinline__ bool mail_try(const MailSlot *s, unsigned long long epoch, float &x) {
    const unsigned long long a = load_agent(&s->w0), b = load_agent(&s->w1);
    x = __uint_as_float((unsigned)a);
    return (a >> 32) == (epoch & 0xffffffffull) && (b >> 32) == (((epoch >> 32) ^ kMailSalt) & 0xffffffffull) &&
           (unsigned)a == (unsigned)b;
}

// On entry s_val holds this part's values at its keys (j < L, j % 4 == part); on return it holds the values of all
// keys below L.  mail_b: the sample's boxes [SP_PARTS receivers][SP_KEYS].  Called by every thread of the block;
// returns false if a value did not arrive in time.
__device__ __forceinline__ bool exchange_over_parts(float *s_val, int *s_ok, MailSlot *mail_b, int part, int L,
                                                    unsigned long long epoch, int lane, int w) {
    lds_barrier();
    if (w == 0) {
        {   // lane = 16 r + i: key part + 4 i to receiver r
            const int i = lane & 15, r = lane >> 4, j = part + SP_PARTS * i;
            if (r != part && j < L) mail_put(&mail_b[r * SP_KEYS + j], s_val[j], epoch);
        }
        bool ok = true;
        if (lane < L && (lane & (SP_PARTS - 1)) != part) {
            MailSlot *s = &mail_b[part * SP_KEYS + lane];
            const long long t0 = wall_clock64();
            float x;
            while (!mail_try(s, epoch, x)) {
                __builtin_amdgcn_s_sleep(1);
                if (wall_clock64() - t0 > kSpinLimitTicks) {
                    ok = false;
                    break;
                }
            }
            s_val[lane] = x;
            store_agent(&s->w0, 0ull);
            store_agent(&s->w1, 0ull);
        }
        const int all_ok = __all(ok) ? 1 : 0;
        if (lane == 0) *s_ok = all_ok;
    }
    lds_barrier();
    return *s_ok != 0;
}

// Forward step.  grid (4, B).  Before the exchange wave w takes the keys part + 4 (w + 8 u) with the lanes along
// h; after it thread (g, c) = (tid / 128, tid % 128) takes the value rows g, g + 4, .. at column part * cw + c.
// The loads that do not depend on the sample's length leave first, then, once key_len is known, every row of a
// valid key at once (rows of masked keys are never read: measured, waiting for the length costs nothing next to
// the 40 % of the bytes it saves at lengths of 10 to 50 out of 50).
template <typename T>
__global__ __launch_bounds__(SP_THREADS) void k_step_fwd_split(
    const T *__restrict__ Qp, const T *__restrict__ Kp, const T *__restrict__ V, const T *__restrict__ v,
    const int *__restrict__ key_len, float *__restrict__ C, float *__restrict__ P, MailSlot *__restrict__ mail,
    unsigned long long epoch, int Tk, int H, int Dv, int cw) {
    __shared__ float s_s[SP_KEYS];
    __shared__ float s_c[SP_GROUPS][SP_COLS];
    __shared__ int s_ok;
    const int part = blockIdx.x, b = blockIdx.y;
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane(wave_id());
    const T *qb = Qp + (size_t)b * H;
    const T *Kb = Kp + (size_t)b * Tk * H;
    const T *Vb = V + (size_t)b * Tk * Dv;

    // ---- every request of the step before the first result is awaited
    const int len_raw = key_len[b];
    float4 q4[SP_CH], v4[SP_CH], k4[SP_CH][SP_KU];
#pragma unroll
    for (int c = 0; c < SP_CH; ++c) {
        if (256 * c < H) {                                        // block-uniform
            const int h = 256 * c + 4 * lane;
            const int hc = min(h, H - 4);
            q4[c] = ld4(qb, (size_t)hc);
            v4[c] = ld4(v, (size_t)hc);
            if (h >= H) v4[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    const int g = w >> 1;                                         // threadIdx.x / SP_COLS, the same in the whole wave
    const int cc = threadIdx.x & (SP_COLS - 1);
    const int d = part * cw + cc;
    const bool d_valid = cc < cw && d < Dv;
    const int d_cl = min(d, Dv - 1);
    const int L = clamp_len(len_raw, Tk);
#pragma unroll
    for (int c = 0; c < SP_CH; ++c) {
        if (256 * c < H) {
            const int hc = min(256 * c + 4 * lane, H - 4);
#pragma unroll
            for (int u = 0; u < SP_KU; ++u) {
                const int j = part + SP_PARTS * (w + SP_W * u);
                if (j < L) k4[c][u] = ld4(Kb, (size_t)j * H + hc);   // wave-uniform: rows of masked keys stay in memory
            }
        }
    }
    float vrow[SP_ROWS];
#pragma unroll
    for (int m = 0; m < SP_ROWS; ++m)
        if (g + SP_GROUPS * m < L) vrow[m] = ld(Vb, (size_t)(g + SP_GROUPS * m) * Dv + d_cl);
    if (L == 0) {                                                 // no valid key (all four parts see that): zeros
        if (g == 0 && d_valid) store_streaming(&C[(size_t)b * Dv + d], 0.f);
        if (part == 0 && w == 1 && lane < Tk) store_streaming(&P[(size_t)b * Tk + lane], 0.f);
        return;
    }

    // ---- scores of this part's keys: S[j] = sum_h v[h] tanh(q[h] + k[j,h]),  tanh = 1 - 2 / (exp(2 (q + k)) + 1)
#pragma unroll
    for (int u = 0; u < SP_KU; ++u) {
        const int j = part + SP_PARTS * (w + SP_W * u);
        if (j < L) {                                              // wave-uniform
            float acc = 0.f;
#pragma unroll
            for (int c = 0; c < SP_CH; ++c) {
                if (256 * c < H) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float x = kTwoLog2e * (comp4s(q4[c], e) + comp4s(k4[c][u], e));
                        acc += comp4s(v4[c], e) * __builtin_fmaf(-2.f, fast_rcp(fast_exp2(x) + 1.0f), 1.0f);
                    }
                }
            }
            const float tot = wave_sum(acc);
            if (lane == 0) s_s[j] = tot;
        }
    }
    const bool ok = exchange_over_parts(s_s, &s_ok, mail + (size_t)b * SP_PARTS * SP_KEYS, part, L, epoch, lane, w);

    // ---- softmax over the valid keys, one key per lane, the same in every wave
    const float sc = lane < L ? s_s[lane] : -INFINITY;
    const float mx = wave_max(sc);
    const float ex = lane < L ? fast_exp2((sc - mx) * 1.4426950408889634f) : 0.f;
    const float z = wave_sum(ex);
    const float p = lane < L ? ex * (1.0f / z) : 0.f;

    // ---- context at this part's columns: the four row groups add their rows, then the groups are added
    float acc = 0.f;
#pragma unroll
    for (int m = 0; m < SP_ROWS; ++m) {
        const int j = g + SP_GROUPS * m;
        if (j < L) acc = __builtin_fmaf(lane_value(p, j), vrow[m], acc);
    }
    s_c[g][cc] = acc;
    lds_barrier();
    const float bad = __builtin_nanf("");
    if (g == 0 && d_valid) {
        const float sum = (s_c[0][cc] + s_c[1][cc]) + (s_c[2][cc] + s_c[3][cc]);
        store_streaming(&C[(size_t)b * Dv + d], ok ? sum : bad);
    }
    if (part == 0 && w == 1 && lane < Tk) store_streaming(&P[(size_t)b * Tk + lane], ok ? p : bad);
}

// Query side of the backward step (key-side sums deferred to the end of the sentence).  grid (4, B).  Before the
// exchange wave w forms dP of the keys part + 4 (w + 8 u) with the lanes along the value columns; after it thread
// (g, c) re-evaluates tanh at the keys g, g + 4, .. and h = part * hw + c.  Writes dQp, and part 0 writes the
// step's row of dS (zeros at masked keys and pads) and its sum.
template <typename T>
__global__ __launch_bounds__(SP_THREADS) void k_step_bwd_query_split(
    const float *__restrict__ dC, const float *__restrict__ P, const T *__restrict__ Qp, const T *__restrict__ Kp,
    const T *__restrict__ V, const T *__restrict__ v, const int *__restrict__ key_len, float *__restrict__ dQp,
    float *__restrict__ ds_out, float *__restrict__ ds_sum_out, int ds_rows, int ds_row, int ds_pitch,
    MailSlot *__restrict__ mail, unsigned long long epoch, int Tk, int H, int Dv, int hw) {
    __shared__ float s_dp[SP_KEYS];
    __shared__ float s_q[SP_GROUPS][SP_COLS];
    __shared__ int s_ok;
    const int part = blockIdx.x, b = blockIdx.y;
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane(wave_id());
    const float *dCb = dC + (size_t)b * Dv;
    const T *Vb = V + (size_t)b * Tk * Dv;
    const T *Kb = Kp + (size_t)b * Tk * H;

    // ---- every request of the step
    const int len_raw = key_len[b];
    const float p_raw = lane < Tk ? P[(size_t)b * Tk + lane] : 0.f;
    float4 c4[SP_CH], x4[SP_CH][SP_KU];
#pragma unroll
    for (int c = 0; c < SP_CH; ++c) {
        if (256 * c < Dv) {                                       // block-uniform
            const int d = 256 * c + 4 * lane;
            const int dc = min(d, Dv - 4);
            c4[c] = ld4(dCb, (size_t)dc);
            if (d >= Dv) c4[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    const int g = w >> 1;
    const int cc = threadIdx.x & (SP_COLS - 1);
    const int h = part * hw + cc;
    const bool h_valid = cc < hw && h < H;
    const int h_cl = min(h, H - 1);
    const float sq = kTwoLog2e * ld(Qp, (size_t)b * H + h_cl);
    const float v4 = 4.f * ld(v, (size_t)h_cl);
    const int L = clamp_len(len_raw, Tk);
#pragma unroll
    for (int c = 0; c < SP_CH; ++c) {
        if (256 * c < Dv) {
            const int dc = min(256 * c + 4 * lane, Dv - 4);
#pragma unroll
            for (int u = 0; u < SP_KU; ++u) {
                const int j = part + SP_PARTS * (w + SP_W * u);
                if (j < L) x4[c][u] = ld4(Vb, (size_t)j * Dv + dc);   // wave-uniform: rows of masked keys stay in memory
            }
        }
    }
    float krow[SP_ROWS];
#pragma unroll
    for (int m = 0; m < SP_ROWS; ++m)
        if (g + SP_GROUPS * m < L) krow[m] = ld(Kb, (size_t)(g + SP_GROUPS * m) * H + h_cl);
    float *ds_dst = ds_out + ((size_t)b * ds_rows + ds_row) * ds_pitch;
    if (L == 0) {                             // no valid key: the query gets no gradient, the stored row is zero
        if (g == 0 && h_valid) store_streaming(&dQp[(size_t)b * H + h], 0.f);
        if (part == 0 && w == 1) {
            if (lane < ds_pitch) ds_dst[lane] = 0.f;
            if (lane == 0) ds_sum_out[(size_t)b * ds_rows + ds_row] = 0.f;
        }
        return;
    }

    // ---- dP[j] = sum_d dC[d] V[j,d] at this part's keys
#pragma unroll
    for (int u = 0; u < SP_KU; ++u) {
        const int j = part + SP_PARTS * (w + SP_W * u);
        if (j < L) {                                              // wave-uniform
            float acc = 0.f;
#pragma unroll
            for (int c = 0; c < SP_CH; ++c)
                if (256 * c < Dv)
                    acc += (c4[c].x * x4[c][u].x + c4[c].y * x4[c][u].y) + (c4[c].z * x4[c][u].z + c4[c].w * x4[c][u].w);
            const float tot = wave_sum(acc);
            if (lane == 0) s_dp[j] = tot;
        }
    }
    const bool ok = exchange_over_parts(s_dp, &s_ok, mail + (size_t)b * SP_PARTS * SP_KEYS, part, L, epoch, lane, w);

    // ---- dS = P (dP - sum_j P dP), one key per lane, the same in every wave
    const float pj = lane < L ? p_raw : 0.f;
    const float dp = lane < L ? s_dp[lane] : 0.f;
    const float r = wave_sum(pj * dp);
    const float ds = pj * (dp - r);
    const float dsum = wave_sum(ds);      // zero in exact arithmetic; kept so that the key-side sums are exact in fp32

    // ---- recomputation at (this group's keys, this thread's h):  r' = 1 / (exp(2 (q + k)) + 1),
    //      1 - t^2 = 4 r' (1 - r');  dQp[h] = v[h] sum_j dS[j] (1 - t^2)
    float accQ = 0.f;
#pragma unroll
    for (int m = 0; m < SP_ROWS; ++m) {
        const int j = g + SP_GROUPS * m;
        if (j < L) {
            const float rr = fast_rcp(fast_exp2(__builtin_fmaf(kTwoLog2e, krow[m], sq)) + 1.0f);
            accQ = __builtin_fmaf(lane_value(ds, j), __builtin_fmaf(-rr, rr, rr), accQ);
        }
    }
    s_q[g][cc] = accQ;
    lds_barrier();
    const float bad = __builtin_nanf("");
    if (g == 0 && h_valid) {
        const float tq = (s_q[0][cc] + s_q[1][cc]) + (s_q[2][cc] + s_q[3][cc]);
        store_streaming(&dQp[(size_t)b * H + h], ok ? v4 * tq : bad);
    }
    if (part == 0 && w == 1) {
        if (lane < ds_pitch) ds_dst[lane] = ok ? ds : bad;
        if (lane == 0) ds_sum_out[(size_t)b * ds_rows + ds_row] = ok ? dsum : bad;
    }
}

// ---- host side ------------------------------------------------------------------------------------------------

static bool split_shape_ok(const AttnShape &s) {
    return s.Tq == 1 && s.Tk <= SP_KEYS && s.H % 4 == 0 && s.H >= 4 && s.H <= SP_MAX_WIDTH && s.Dv % 4 == 0 &&
           s.Dv >= 4 && s.Dv <= SP_MAX_WIDTH && s.B <= kStepSplitMaxB;
}

size_t step_split_mail_bytes(const AttnShape &s) {
    return split_shape_ok(s) ? (size_t)s.B * SP_PARTS * SP_KEYS * sizeof(MailSlot) : 0;
}

// The four blocks of a sample wait for one another: the form is used only where all 4 B blocks run at once, one
// per compute unit.  The number of compute units is asked once per device.
bool step_split_applicable(const AttnShape &s) {
    if (!split_shape_ok(s)) return false;
    static std::atomic<int> cu_count[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return false;
    int n = cu_count[dev].load(std::memory_order_acquire);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return false;
        cu_count[dev].store(n, std::memory_order_release);
    }
    return SP_PARTS * s.B <= n;
}

hipError_t launch_step_fwd_split(const AttnShape &s, const void *Qp, const void *Kp, const void *V, const void *v,
                                 const int *key_len, float *C, float *P, void *mail, unsigned long long epoch,
                                 hipStream_t st) {
    if (!split_shape_ok(s) || !mail || epoch == 0) return hipErrorInvalidValue;
    const int cw = (s.Dv + SP_PARTS - 1) / SP_PARTS;
    dim3 grid(SP_PARTS, s.B);
    if (s.bf16)
        k_step_fwd_split<bf16_t><<<grid, SP_THREADS, 0, st>>>((const bf16_t *)Qp, (const bf16_t *)Kp, (const bf16_t *)V,
                                                              (const bf16_t *)v, key_len, C, P, (MailSlot *)mail, epoch,
                                                              s.Tk, s.H, s.Dv, cw);
    else
        k_step_fwd_split<float><<<grid, SP_THREADS, 0, st>>>((const float *)Qp, (const float *)Kp, (const float *)V,
                                                             (const float *)v, key_len, C, P, (MailSlot *)mail, epoch,
                                                             s.Tk, s.H, s.Dv, cw);
    return hipGetLastError();
}

hipError_t launch_step_bwd_query_split(const AttnShape &s, const float *dC, const float *P, const void *Qp,
                                       const void *Kp, const void *V, const void *v, const int *key_len, float *dQp,
                                       float *ds_out, float *ds_sum_out, int steps, int step, void *mail,
                                       unsigned long long epoch, hipStream_t st) {
    if (!split_shape_ok(s) || !mail || epoch == 0) return hipErrorInvalidValue;
    const int hw = (s.H + SP_PARTS - 1) / SP_PARTS;
    dim3 grid(SP_PARTS, s.B);
    if (s.bf16)
        k_step_bwd_query_split<bf16_t><<<grid, SP_THREADS, 0, st>>>(
            dC, P, (const bf16_t *)Qp, (const bf16_t *)Kp, (const bf16_t *)V, (const bf16_t *)v, key_len, dQp, ds_out,
            ds_sum_out, steps, step, ds_pitch(s.Tk), (MailSlot *)mail, epoch, s.Tk, s.H, s.Dv, hw);
    else
        k_step_bwd_query_split<float><<<grid, SP_THREADS, 0, st>>>(
            dC, P, (const float *)Qp, (const float *)Kp, (const float *)V, (const float *)v, key_len, dQp, ds_out,
            ds_sum_out, steps, step, ds_pitch(s.Tk), (MailSlot *)mail, epoch, s.Tk, s.H, s.Dv, hw);
    return hipGetLastError();
}

}  // namespace echo
