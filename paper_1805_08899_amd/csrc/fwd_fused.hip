// Forward pass in one kernel: scores, masked softmax and context for a tile of
// query rows of one sample, without S ever reaching memory
// (Section 2, attention steps 1-2; Section 4.1 scoring function; Section 6.1:
// one fused kernel instead of many small ones, fewer launches and accesses).
//
// Block = (sample b, FW_R query rows), 8 waves, two blocks per CU.
//   A  exp(2q) and 2 log2e q of the rows go to LDS (taken once per block).
//   B  keys are dealt to the waves round-robin, FW_RJ per wave and chunk of 32;
//      lanes run along h.  A wave loads its own key rows straight from memory
//      (every K element is exponentiated once per block), evaluates its rows x
//      keys register tile slice by slice of 64 h
//          acc += v[h] * rcp(fma(exp(2q), exp(2k), 1))
//      and finishes with one transposing wave reduction per tile.
//   C  wave r normalises row r (softmax over the valid keys), writes P.
//   D  context = P V on the matrix cores: v_mfma_f32_4x4x1 treats the 64 lanes
//      as 16 column groups of 4, so a lane owns one output column and reads V
//      rows with plain coalesced loads.
//
// The whole pass of a block is short compared with a trip to memory, so every
// phase issues its loads in deep batches before it consumes them, and nothing
// that is loaded first depends on key_len: query rows and the first key slices
// leave before anything is waited for, key slices run FW_PF ahead of the
// arithmetic, and the first FW_KB value rows leave before the softmax.
//
// Two 8-wave blocks share a CU, so a CU works through the sum of its two
// tiles at full rate whatever their mix of key lengths.  The tiles of one
// sample share an XCD (and its L2).
#include "common.hpp"
#include "kernels.hpp"

namespace echo {

typedef float f32x4 __attribute__((ext_vector_type(4)));

#ifdef ECHO_TIMING   // development aid: per-block phase time stamps (100 MHz counter), read back with echo_debug_stamps
__device__ long long g_stamps[16384 * 8];
#define FW_STAMP(k)                                                                                 \
    do {                                                                                            \
        if (threadIdx.x == 0 && blockIdx.x < 16384) g_stamps[blockIdx.x * 8 + (k)] = wall_clock64(); \
    } while (0)
#else
#define FW_STAMP(k)
#endif

constexpr int FW_R = 8;          // query rows per block (register tile rows)
constexpr int FW_RJ = 4;         // keys per wave and chunk (register tile columns)
constexpr int FW_W = 8;          // waves per block
constexpr int FW_CHUNK = FW_W * FW_RJ;   // keys per chunk
constexpr int FW_THREADS = 64 * FW_W;
constexpr int FW_XCD = 8;        // blockIdx.x mod 8 selects the XCD
constexpr int FW_PF = 4;         // slices of h whose key values are in flight per wave
constexpr int FW_KB = 32;        // value rows in flight per wave in the context phase

// One wave, NJ keys (rows krow0 + c*kstride), all slices of h.  s_e / s_s: LDS rows of exp(2q) /
// 2 log2e q, pitch Hp.  FULL: all FW_R rows are live, else the first ni.  kx[u][c] / vx[u] arrive
// holding slices 0..FW_PF-1 of the wave's keys and of v (invalid lanes of v hold 0) and are
// refilled FW_PF slices ahead.
template <typename T, int NJ, bool FULL>
__device__ __forceinline__ void fw_score_wave(const float *__restrict__ s_e, const float *__restrict__ s_s, int Hp,
                                              int ni, bool qbig, const T *__restrict__ krow0, size_t kstride, int H,
                                              const T *__restrict__ v, float *__restrict__ s_S, int spitch,
                                              int jcol0, float (&kx)[FW_PF][FW_RJ], float (&vx)[FW_PF]) {
    const int lane = lane_id();
    float acc[FW_R][NJ];
#pragma unroll
    for (int a = 0; a < FW_R; ++a)
#pragma unroll
        for (int c = 0; c < NJ; ++c) acc[a][c] = 0.f;
    float vsum = 0.f;
    const int nsl = (H + 63) / 64;

    for (int s0 = 0; s0 < nsl; s0 += FW_PF) {
#ifdef ECHO_TIMING
        if (s0 == FW_PF && jcol0 < FW_W) FW_STAMP(1);
#endif
#pragma unroll
        for (int u = 0; u < FW_PF; ++u) {
            const int sl = s0 + u;
            if (sl < nsl) {
                const int h0 = sl * 64;
                const float vh = vx[u];
                const bool hv = h0 + lane < H;
                bool kbig = false;
                float fk[NJ];                 // 2 log2e k of this slice; turned into exp(2k) on the factor path
#pragma unroll
                for (int c = 0; c < NJ; ++c) {
                    const float x = hv ? kx[u][c] : 0.f;
                    kbig |= fabsf(x) > kFactorLimit;
                    fk[c] = kTwoLog2e * x;
                }
#ifdef ECHO_TIMING
                if (sl == 0 && jcol0 < FW_W) {
                    asm volatile("" ::"v"(fk[0]), "v"(vh));
                    FW_STAMP(2);
                }
#endif
                if (sl + FW_PF < nsl) {       // refill this ring slot
                    const int hn = h0 + FW_PF * 64 + lane;
                    const int hc = hn < H ? hn : H - 1;
#pragma unroll
                    for (int c = 0; c < NJ; ++c) kx[u][c] = ld(krow0, (size_t)c * kstride + hc);
                    vx[u] = hn < H ? ld(v, hc) : 0.f;
                }
                vsum += vh;
                const bool exact = qbig || __any(kbig);
                const float *qrow = (exact ? s_s : s_e) + h0 + lane;
                float fq[FW_R];               // rows past ni hold zeros in LDS
#pragma unroll
                for (int a = 0; a < FW_R; ++a) fq[a] = qrow[a * Hp];
                if (!exact) {
#pragma unroll
                    for (int c = 0; c < NJ; ++c) fk[c] = fast_exp2(fk[c]);
#pragma unroll
                    for (int a = 0; a < FW_R; ++a) {
                        if (FULL || a < ni) {
#pragma unroll
                            for (int c = 0; c < NJ; ++c)
                                acc[a][c] = __builtin_fmaf(vh, r_from_factors(fq[a], fk[c]), acc[a][c]);
                        }
                    }
                } else {
#pragma unroll
                    for (int a = 0; a < FW_R; ++a) {
                        if (FULL || a < ni) {
#pragma unroll
                            for (int c = 0; c < NJ; ++c)
                                acc[a][c] = __builtin_fmaf(vh, r_from_sum(fq[a], fk[c]), acc[a][c]);
                        }
                    }
                }
            }
        }
    }
#ifdef ECHO_TIMING
    if (jcol0 < FW_W) FW_STAMP(5);
#endif
    // S = sum_h v (1 - 2r): per lane first, then one transposing reduction for the whole tile
    constexpr int NP = FW_R * NJ;
    constexpr int NPOW = NP <= 8 ? 8 : NP <= 16 ? 16 : NP <= 32 ? 32 : 64;
    float flat[NPOW];
#pragma unroll
    for (int p = 0; p < NPOW; ++p) {
        const int a = p / NJ, c = p % NJ;
        flat[p] = p < NP ? __builtin_fmaf(-2.f, acc[a < FW_R ? a : 0][c], vsum) : 0.f;
    }
    const float tot = wave_transpose_sum<NPOW>(flat);
    const int p = lane / (64 / NPOW);
    if ((lane % (64 / NPOW)) == 0 && p < NP) {
        const int a = p / NJ, c = p % NJ;
        if (a < ni && jcol0 + c * FW_W < spitch - 4) s_S[a * spitch + jcol0 + c * FW_W] = tot;
    }
}

template <typename T>
__global__ __launch_bounds__(FW_THREADS, 4) void k_fwd_fused(
    const T *__restrict__ Qp, const T *__restrict__ Kp, const T *__restrict__ V, const T *__restrict__ v,
    const int *__restrict__ key_len, float *__restrict__ C, float *__restrict__ P,
    int B, int Tq, int Tk, int H, int Dv, int tiles, int Hp, int spitch) {
    extern __shared__ float smem[];
    float *s_e = smem;                       // [FW_R][Hp]  exp(2q)
    float *s_s = s_e + FW_R * Hp;            // [FW_R][Hp]  2 log2e q
    float *s_S = s_s + FW_R * Hp;            // [FW_R][spitch]  scores, then probabilities

    const int lane = lane_id(), w = wave_id();
    FW_STAMP(0);

    // ---- which (sample, row tile): XCD x takes samples x, x+8, ...
    const int xcd = blockIdx.x % FW_XCD, idx = blockIdx.x / FW_XCD;
    const int b = xcd + FW_XCD * (idx / tiles), tile = idx % tiles;
    if (b >= B) return;
    const int r0 = tile * FW_R;
    const int ni = min(FW_R, Tq - r0);                        // 1..FW_R

    // ---- loads that do not depend on key_len go out first: the query rows ...
    const T *qb = Qp + ((size_t)b * Tq + r0) * H;
    constexpr int QMAX = 2;                                   // column passes per batch (H <= 1024 in one batch)
    float qx[QMAX][FW_R];
    auto q_fetch = [&](int col0) {
#pragma unroll
        for (int m = 0; m < QMAX; ++m) {
            const int h = col0 + m * FW_THREADS + threadIdx.x;
#pragma unroll
            for (int a = 0; a < FW_R; ++a) qx[m][a] = (a < ni && h < H) ? ld(qb, (size_t)a * H + h) : 0.f;
        }
    };
    q_fetch(0);

    // ... and the first FW_PF slices of this wave's keys of chunk 0.  Wave w owns keys
    // 32 ch + 8 c + w (c < FW_RJ) of chunk ch; rows past Tk are clamped and never used.
    const T *kb = Kp + (size_t)b * Tk * H;
    const int nsl = (H + 63) / 64;
    float kx[FW_PF][FW_RJ], vx[FW_PF];
    auto k_prefetch = [&](int ch) {
#pragma unroll
        for (int u = 0; u < FW_PF; ++u) {
            const int hn = u * 64 + lane;
            const int hc = hn < H ? hn : H - 1;
            const bool on = u < nsl;
#pragma unroll
            for (int c = 0; c < FW_RJ; ++c) {
                const int j = min(ch * FW_CHUNK + c * FW_W + w, Tk - 1);
                kx[u][c] = on ? ld(kb, (size_t)j * H + hc) : 0.f;
            }
            vx[u] = (on && hn < H) ? ld(v, hc) : 0.f;
        }
    };
    k_prefetch(0);

    const int L = clamp_len(key_len[b], Tk);
    float *Pb = P + ((size_t)b * Tq + r0) * Tk;
    float *Cb = C + ((size_t)b * Tq + r0) * Dv;
    if (L == 0) {                                             // no valid key: zeros
        for (int e = threadIdx.x; e < ni * Tk; e += FW_THREADS) Pb[e] = 0.f;
        for (int e = threadIdx.x; e < ni * Dv; e += FW_THREADS) Cb[e] = 0.f;
        return;
    }

    // ---- A: exp(2q) and 2 log2e q to LDS (rows past ni and columns past H as zeros)
    bool big = false;
    for (int col0 = 0; col0 < Hp; col0 += QMAX * FW_THREADS) {
        if (col0 > 0) q_fetch(col0);
#pragma unroll
        for (int m = 0; m < QMAX; ++m) {
            const int h = col0 + m * FW_THREADS + threadIdx.x;
            if (h < Hp) {
#pragma unroll
                for (int a = 0; a < FW_R; ++a) {
                    big |= fabsf(qx[m][a]) > kFactorLimit;
                    const float sc = kTwoLog2e * qx[m][a];
                    s_s[a * Hp + h] = sc;
                    s_e[a * Hp + h] = (a < ni && h < H) ? fast_exp2(sc) : 0.f;
                }
            }
        }
    }
    const bool qbig = __syncthreads_or(big) != 0;
    FW_STAMP(3);

    // ---- B: scores, keys in chunks of FW_CHUNK
    const int n_chunk = (L + FW_CHUNK - 1) / FW_CHUNK;
    for (int ch = 0; ch < n_chunk; ++ch) {
        if (ch > 0) k_prefetch(ch);
        const int j0 = ch * FW_CHUNK + w;                      // first key of this wave in the chunk
        const int nj = j0 < L ? min(FW_RJ, (L - 1 - j0) / FW_W + 1) : 0;
        const T *krow0 = kb + (size_t)j0 * H;
        const size_t kstride = (size_t)FW_W * H;
#define FW_CASE(N)                                                                                              \
    case N:                                                                                                     \
        if (ni == FW_R)                                                                                         \
            fw_score_wave<T, N, true>(s_e, s_s, Hp, ni, qbig, krow0, kstride, H, v, s_S, spitch, j0, kx, vx);   \
        else                                                                                                    \
            fw_score_wave<T, N, false>(s_e, s_s, Hp, ni, qbig, krow0, kstride, H, v, s_S, spitch, j0, kx, vx);  \
        break;
#ifdef FW_ONE_VARIANT
        if (nj > 0) fw_score_wave<T, 4, false>(s_e, s_s, Hp, ni, qbig, krow0, kstride, H, v, s_S, spitch, j0, kx, vx);
#else
        switch (nj) {
            FW_CASE(1) FW_CASE(2) FW_CASE(3) FW_CASE(4)
            default: break;
        }
#endif
#undef FW_CASE
    }

    // first batch of value rows for the context phase leaves before the softmax
    const T *vb = V + (size_t)b * Tk * Dv;
    const int Lp = (L + 3) & ~3;
    const int n_grp = (Dv + 63) / 64;
    float vv[FW_KB];
    auto v_fetch = [&](int g, int kb0) {
        const int n = g * 64 + lane;
        const int nc = n < Dv ? n : Dv - 1;
#pragma unroll
        for (int kk = 0; kk < FW_KB; ++kk)   // keys past L carry P = 0; the last valid row stands in for them
            if (kb0 + kk < Lp) vv[kk] = ld(vb, (size_t)min(kb0 + kk, L - 1) * Dv + nc);
    };
    if (w < n_grp) v_fetch(w, 0);
    __syncthreads();
    FW_STAMP(4);

    // ---- C: softmax, wave r <-> row r; probabilities replace the scores in LDS
    for (int a = w; a < FW_R; a += FW_W) {
        float *srow = s_S + a * spitch;
        if (a < ni) {
            float m = -INFINITY;
            for (int j = lane; j < L; j += 64) m = fmaxf(m, srow[j]);
            m = wave_max(m);
            float z = 0.f;
            for (int j = lane; j < L; j += 64) {
                const float e = fast_exp2((srow[j] - m) * 1.4426950408889634f);
                srow[j] = e;
                z += e;
            }
            z = wave_sum(z);
            const float inv = 1.0f / z;
            for (int j = lane; j < max(Tk, Lp); j += 64) {
                const float p = j < L ? srow[j] * inv : 0.f;
                if (j < Lp) srow[j] = p;
                if (j < Tk) Pb[(size_t)a * Tk + j] = p;
            }
        } else {
            for (int j = lane; j < Lp; j += 64) srow[j] = 0.f;
        }
    }
    __syncthreads();

    // ---- D: context rows = P V.  A wave takes 64 columns at a time; lane l owns column n0 + l.
    // One 4x4x1 MFMA multiplies 4 rows of P (replicated over the 16 lane groups) with one V value per lane.
    const int lr = lane & 3;
    for (int g = w; g < n_grp; g += FW_W) {
        const int n = g * 64 + lane;
        f32x4 a0 = {0.f, 0.f, 0.f, 0.f}, a1 = a0;              // rows 0-3 / 4-7
        for (int kb0 = 0; kb0 < Lp; kb0 += FW_KB) {
            if (g != w || kb0 > 0) v_fetch(g, kb0);
#pragma unroll
            for (int k4 = 0; k4 < FW_KB; k4 += 4) {
                if (kb0 + k4 < Lp) {
                    const float4 pa = *reinterpret_cast<const float4 *>(s_S + lr * spitch + kb0 + k4);
                    const float4 pb = *reinterpret_cast<const float4 *>(s_S + (4 + lr) * spitch + kb0 + k4);
                    const float pav[4] = {pa.x, pa.y, pa.z, pa.w}, pbv[4] = {pb.x, pb.y, pb.z, pb.w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        a0 = __builtin_amdgcn_mfma_f32_4x4x1f32(pav[q], vv[k4 + q], a0, 0, 0, 0);
                        a1 = __builtin_amdgcn_mfma_f32_4x4x1f32(pbv[q], vv[k4 + q], a1, 0, 0, 0);
                    }
                }
            }
        }
        if (n < Dv) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (r < ni) Cb[(size_t)r * Dv + n] = a0[r];
                if (4 + r < ni) Cb[(size_t)(4 + r) * Dv + n] = a1[r];
            }
        }
    }
    FW_STAMP(6);
#ifdef ECHO_TIMING
    if (threadIdx.x == 0 && blockIdx.x < 16384) {
        unsigned hw, xcc;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        g_stamps[blockIdx.x * 8 + 7] = ((long long)xcc << 32) | hw;
    }
#endif
}

#ifdef ECHO_TIMING
extern "C" int echo_debug_stamps(long long *host, int n) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_stamps), (size_t)n * sizeof(long long));
}
#endif

size_t fwd_fused_lds_bytes(const AttnShape &s) {
    const int Hp = (s.H + 63) / 64 * 64;
    const int spitch = ((s.Tk + 3) & ~3) + 4;
    return (size_t)(2 * FW_R * Hp + FW_R * spitch) * sizeof(float);
}

template <typename T>
static hipError_t launch_fwd_fused_t(const AttnShape &s, const void *Qp, const void *Kp, const void *V, const void *v,
                                     const int *key_len, float *C, float *P, hipStream_t st) {
    const int Hp = (s.H + 63) / 64 * 64;
    const int spitch = ((s.Tk + 3) & ~3) + 4;
    const size_t lds = fwd_fused_lds_bytes(s);
    static size_t attr_bytes = 48 * 1024;   // dynamic LDS limit already granted to this instantiation
    if (lds > attr_bytes) {
        hipError_t e = hipFuncSetAttribute((const void *)k_fwd_fused<T>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds);
        if (e != hipSuccess) return e;
        attr_bytes = lds;
    }
    const int tiles = (s.Tq + FW_R - 1) / FW_R;
    const int samples_per_xcd = (s.B + FW_XCD - 1) / FW_XCD;
    const int grid = FW_XCD * samples_per_xcd * tiles;
    k_fwd_fused<T><<<grid, FW_THREADS, lds, st>>>((const T *)Qp, (const T *)Kp, (const T *)V, (const T *)v, key_len, C,
                                                  P, s.B, s.Tq, s.Tk, s.H, s.Dv, tiles, Hp, spitch);
    return hipGetLastError();
}

hipError_t launch_fwd_fused(const AttnShape &s, const void *Qp, const void *Kp, const void *V, const void *v,
                            const int *key_len, float *C, float *P, hipStream_t st) {
    return s.bf16 ? launch_fwd_fused_t<bf16_t>(s, Qp, Kp, V, v, key_len, C, P, st)
                  : launch_fwd_fused_t<float>(s, Qp, Kp, V, v, key_len, C, P, st);
}

}  // namespace echo
