// Forward pass in one kernel: scores, masked softmax and context for a tile of
// query rows of one sample, without S ever reaching memory
// (Section 2, attention steps 1-2; Section 4.1 scoring function; Section 6.1:
// one fused kernel instead of many small ones, fewer launches and accesses).
//
// Block = (sample b, FW_R query rows), 8 waves, two blocks per CU.
//   A  exp(2q) of the rows goes to LDS (taken once per block).
//   B  keys are dealt to the waves round-robin, FW_RJ per wave and chunk of 32;
//      lanes run along h.  A wave loads its own key rows straight from memory
//      (every K element is exponentiated once per block), evaluates its rows x
//      keys register tile slice by slice of 64 h
//          acc += v[h] * rcp(fma(exp(2q), exp(2k), 1))
//      and finishes with one transposing wave reduction per tile.  A tile that
//      met a pre-activation beyond the factorisation limit is redone by a
//      small exact routine that exponentiates the sum.
//   C  wave r normalises row r (softmax over the valid keys), writes P.
//   D  context = P V on the matrix cores: v_mfma_f32_4x4x1 treats the 64 lanes
//      as 16 column groups of 4, so a lane owns one output column and reads V
//      rows with plain coalesced loads.
//
// The whole pass of a block is short compared with a trip to memory, so every
// phase issues its loads in batches before it consumes them: query rows and
// the first key slices leave together, key slices run FW_PF ahead of the
// arithmetic, and the first FW_KB value rows leave before the softmax.
//
// Placement.  Two 8-wave blocks share a CU; the hardware hands blocks to the
// XCDs round-robin and, while every block of the grid fits at once, block i
// and block i + 256 land on the same CU.  The kernel ranks the samples by
// valid keys, deals them to the XCDs in snake order (equal work per XCD, and
// all tiles of a sample share one L2), and inside an XCD gives the CUs that
// hold one block the heaviest tiles and pairs heavy with light tiles on the
// others.  With more than two rounds of blocks it simply starts the heaviest
// first.  The mapping only moves work around; results do not depend on it.
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
constexpr int FW_CU_PER_XCD = 32;
constexpr int FW_PF = 4;         // slices of h whose key values are in flight per wave
constexpr int FW_KB = 32;        // value rows in flight per wave in the context phase
constexpr int FW_MAX_RANKED_B = 1024;   // the in-kernel ranking is quadratic in B

// One wave, NJ keys (rows krow0 + c*kstride), all slices of h, factor path only.  s_e: LDS rows of
// exp(2q), pitch Hp (rows past ni hold zeros).  FULL: all FW_R rows are live, else the first ni.
// kx[u][c] / vx[u] arrive holding slices 0..FW_PF-1 of the wave's keys and of v (invalid lanes of v
// hold 0); the ring is rotated every slice and refilled FW_PF slices ahead.  Returns true if a key value was beyond the factor
// limit, in which case nothing was written and the caller must redo the tile exactly.
template <typename T, int NJ, bool FULL>
__device__ __forceinline__ bool fw_score_wave(const float *__restrict__ s_e, int Hp, int ni,
                                              const T *__restrict__ krow0, size_t kstride, int H,
                                              const T *__restrict__ v, float *__restrict__ s_S, int spitch,
                                              int jcol0, float (&kx)[FW_PF][FW_RJ], float (&vx)[FW_PF]) {
    const int lane = lane_id();
    float acc[FW_R][NJ];
#pragma unroll
    for (int a = 0; a < FW_R; ++a)
#pragma unroll
        for (int c = 0; c < NJ; ++c) acc[a][c] = 0.f;
    float vsum = 0.f;
    bool kbig = false;
    const int nsl = (H + 63) / 64;

    for (int sl = 0; sl < nsl; ++sl) {
        const int h0 = sl * 64;
        const float vh = vx[0];
        const bool hv = h0 + lane < H;
        float fk[NJ];
#pragma unroll
        for (int c = 0; c < NJ; ++c) {
            const float x = hv ? kx[0][c] : 0.f;
            kbig |= fabsf(x) > kFactorLimit;
            fk[c] = fast_exp2(kTwoLog2e * x);
        }
        // rotate the ring (the loop stays rolled, so the code stays small) and refill its last slot
#pragma unroll
        for (int u = 0; u + 1 < FW_PF; ++u) {
#pragma unroll
            for (int c = 0; c < NJ; ++c) kx[u][c] = kx[u + 1][c];
            vx[u] = vx[u + 1];
        }
        if (sl + FW_PF < nsl) {
            const int hn = h0 + FW_PF * 64 + lane;
            const int hc = hn < H ? hn : H - 1;
#pragma unroll
            for (int c = 0; c < NJ; ++c) kx[FW_PF - 1][c] = ld(krow0, (size_t)c * kstride + hc);
            vx[FW_PF - 1] = hn < H ? ld(v, hc) : 0.f;
        }
        vsum += vh;
        float fq[FW_R];
#pragma unroll
        for (int a = 0; a < FW_R; ++a) fq[a] = s_e[a * Hp + h0 + lane];
#pragma unroll
        for (int a = 0; a < FW_R; ++a) {
            if (FULL || a < ni) {
#pragma unroll
                for (int c = 0; c < NJ; ++c) acc[a][c] = __builtin_fmaf(vh, r_from_factors(fq[a], fk[c]), acc[a][c]);
            }
        }
    }
    if (__any(kbig)) return true;
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
        if (a < ni) s_S[a * spitch + jcol0 + c * FW_W] = tot;
    }
    return false;
}

// The same tile with tanh taken from the exponential of the sum: correct for any finite input.
// Straightforward loops; only reached for pre-activations beyond the factor limit.
template <typename T>
__device__ __noinline__ void fw_score_wave_exact(const T *__restrict__ qrow0, int ni, const T *__restrict__ krow0,
                                                 size_t kstride, int nj, int H, const T *__restrict__ v,
                                                 float *__restrict__ s_S, int spitch, int jcol0) {
    const int lane = lane_id();
    for (int a = 0; a < ni; ++a) {
        for (int c = 0; c < nj; ++c) {
            float acc = 0.f;
            for (int h = lane; h < H; h += 64) {
                const float sq = kTwoLog2e * ld(qrow0, (size_t)a * H + h);
                const float sk = kTwoLog2e * ld(krow0, (size_t)c * kstride + h);
                const float vh = ld(v, h);
                acc += vh * __builtin_fmaf(-2.f, r_from_sum(sq, sk), 1.f);
            }
            acc = wave_sum(acc);
            if (lane == 0) s_S[a * spitch + jcol0 + c * FW_W] = acc;
        }
    }
}

// Which (sample, row tile) this block works on; see "Placement" at the top.  s_i: scratch of
// 2*B + 2 ints in LDS.  Returns false if the block has nothing to do.
__device__ __forceinline__ bool fw_pick_item(const int *__restrict__ key_len, int B, int Tq, int Tk, int tiles,
                                             int ranked, int *s_i, int &b, int &tile) {
    const int xcd = blockIdx.x % FW_XCD, li = blockIdx.x / FW_XCD;
    if (!ranked) {                         // samples x, x+8, ... on XCD x, in index order
        b = xcd + FW_XCD * (li / tiles);
        tile = li % tiles;
        return b < B;
    }
    int *s_len = s_i, *s_xb = s_i + B, *s_cnt = s_i + 2 * B;
    for (int o = threadIdx.x; o < B; o += FW_THREADS) s_len[o] = clamp_len(key_len[o], Tk);
    if (threadIdx.x == 0) *s_cnt = 0;
    __syncthreads();
    for (int cand = threadIdx.x; cand < B; cand += FW_THREADS) {
        const int lc = s_len[cand];
        int r = 0;                         // rank by valid keys, most first, ties by index
        for (int o = 0; o < B; ++o) {
            const int lo = s_len[o];
            r += (lo > lc) || (lo == lc && o < cand);
        }
        const int q = r % (2 * FW_XCD);
        const int x = q < FW_XCD ? q : 2 * FW_XCD - 1 - q;     // snake over the XCDs
        if (x == xcd) {
            s_xb[(r / (2 * FW_XCD)) * 2 + (q >= FW_XCD ? 1 : 0)] = cand;   // position inside the XCD, heaviest first
            atomicAdd(s_cnt, 1);
        }
    }
    __syncthreads();
    const int M = *s_cnt;                  // samples of this XCD
    const int n = M * tiles;               // its tiles
    if (li >= n) return false;
    // position in the launch order -> position in "heaviest first" order
    int rho = li;
    if (n > FW_CU_PER_XCD && n <= 2 * FW_CU_PER_XCD) {
        const int singles = 2 * FW_CU_PER_XCD - n;             // CUs that get one block: the heaviest tiles
        if (li >= FW_CU_PER_XCD) rho = n - 1 - (li - FW_CU_PER_XCD);
        else if (li >= FW_CU_PER_XCD - singles) rho = li - (FW_CU_PER_XCD - singles);
        else rho = singles + li;
    }
    // heaviest-first list: sample by sample (the tiles of a sample weigh the same)
    const int m = rho / tiles;
    tile = rho % tiles;
    b = s_xb[m];
    return true;
}

template <typename T>
__global__ __launch_bounds__(FW_THREADS, 4) void k_fwd_fused(
    const T *__restrict__ Qp, const T *__restrict__ Kp, const T *__restrict__ V, const T *__restrict__ v,
    const int *__restrict__ key_len, float *__restrict__ C, float *__restrict__ P,
    int B, int Tq, int Tk, int H, int Dv, int tiles, int Hp, int spitch, int ranked) {
    extern __shared__ float smem[];
    float *s_e = smem;                       // [FW_R][Hp]  exp(2q)
    float *s_S = s_e + FW_R * Hp;            // [FW_R][spitch]  scores, then probabilities

    const int lane = lane_id(), w = wave_id();
    FW_STAMP(0);

    int b, tile;
    if (!fw_pick_item(key_len, B, Tq, Tk, tiles, ranked, reinterpret_cast<int *>(smem), b, tile)) return;
    if (ranked) __syncthreads();             // the scratch is about to be overwritten by the staging
    const int r0 = (int)(((long long)Tq * tile) / tiles);      // rows are split evenly over the tiles
    const int ni = (int)(((long long)Tq * (tile + 1)) / tiles) - r0;   // 1..FW_R
    FW_STAMP(1);

    // ---- loads first: the query rows ...
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
#ifdef ECHO_TIMING
    if (threadIdx.x == 0 && blockIdx.x < 16384) g_stamps[blockIdx.x * 8 + 2] = ((long long)b << 40) | ((long long)tile << 24) | ((long long)ni << 16) | L;
#endif

    // ---- A: exp(2q) to LDS (rows past ni and columns past H as zeros)
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
                    s_e[a * Hp + h] = (a < ni && h < H) ? fast_exp2(kTwoLog2e * qx[m][a]) : 0.f;
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
        bool redo = qbig && nj > 0;
        if (!qbig) {
#define FW_CASE(N)                                                                                         \
    case N:                                                                                                \
        redo = (ni == FW_R) ? fw_score_wave<T, N, true>(s_e, Hp, ni, krow0, kstride, H, v, s_S, spitch, j0, kx, vx) \
                            : fw_score_wave<T, N, false>(s_e, Hp, ni, krow0, kstride, H, v, s_S, spitch, j0, kx, vx); \
        break;
            switch (nj) {
                FW_CASE(1) FW_CASE(2) FW_CASE(3) FW_CASE(4)
                default: break;
            }
#undef FW_CASE
        }
        if (redo) fw_score_wave_exact<T>(qb, ni, krow0, kstride, nj, H, v, s_S, spitch, j0);
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
    FW_STAMP(5);

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
    const size_t stage = (size_t)(FW_R * Hp + FW_R * spitch) * sizeof(float);
    const size_t rank_scratch = (size_t)(2 * s.B + 2) * sizeof(int);
    return stage > rank_scratch ? stage : rank_scratch;
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
    const int ranked = s.B <= FW_MAX_RANKED_B ? 1 : 0;
    k_fwd_fused<T><<<grid, FW_THREADS, lds, st>>>((const T *)Qp, (const T *)Kp, (const T *)V, (const T *)v, key_len, C,
                                                  P, s.B, s.Tq, s.Tk, s.H, s.Dv, tiles, Hp, spitch, ranked);
    return hipGetLastError();
}

hipError_t launch_fwd_fused(const AttnShape &s, const void *Qp, const void *Kp, const void *V, const void *v,
                            const int *key_len, float *C, float *P, hipStream_t st) {
    return s.bf16 ? launch_fwd_fused_t<bf16_t>(s, Qp, Kp, V, v, key_len, C, P, st)
                  : launch_fwd_fused_t<float>(s, Qp, Kp, V, v, key_len, C, P, st);
}

}  // namespace echo
