// Forward pass in one kernel: scores, masked softmax and context for a tile of
// query rows of one sample, without S ever reaching memory
// (Section 2, attention steps 1-2; Section 4.1 scoring function; Section 6.1:
// one fused kernel instead of many small ones, fewer launches and accesses).
//
// Block = (sample b, up to FW_R query rows), 4 waves.
//   A  exp(2q) and 2 log2e q of the rows go to LDS (taken once per block).
//   B  the valid keys are dealt to the waves in contiguous runs of at most
//      FW_RJ; lanes run along h.  A wave loads its own key rows straight from
//      memory (every K element is exponentiated once per block), evaluates its
//      rows x keys register tile slice by slice of 64 h
//          acc += v[h] * rcp(fma(exp(2q), exp(2k), 1))
//      and finishes with one transposing wave reduction per tile.
//   C  wave r normalises row r (softmax over the valid keys), writes P.
//   D  context = P V on the matrix cores: v_mfma_f32_4x4x1 treats the 64 lanes
//      as 16 column groups of 4, so a lane owns one output column and reads V
//      rows with plain coalesced loads.
//
// Blocks are ordered so that the samples with the most valid keys start
// first and the tiles of one sample share an XCD (and its L2).
#include "common.hpp"
#include "kernels.hpp"

namespace echo {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int FW_R = 8;          // query rows per block (register tile rows)
constexpr int FW_RJ = 8;         // keys per wave and chunk (register tile columns)
constexpr int FW_W = 4;          // waves per block (one per SIMD; three blocks share a CU)
constexpr int FW_THREADS = 64 * FW_W;
constexpr int FW_XCD = 8;        // blockIdx.x mod 8 selects the XCD

// One wave, NJ keys, all slices of h.  s_e / s_s: LDS rows of exp(2q) / 2 log2e q, pitch Hp.
template <typename T, int NJ>
__device__ __forceinline__ void fw_score_wave(const float *__restrict__ s_e, const float *__restrict__ s_s, int Hp,
                                              int ni, bool qbig, const T *__restrict__ krow0, int H,
                                              const T *__restrict__ v, float *__restrict__ s_S, int spitch,
                                              int jcol0, const float (&kx0)[FW_RJ], float vx0) {
    const int lane = lane_id();
    float acc[FW_R][NJ];
#pragma unroll
    for (int a = 0; a < FW_R; ++a)
#pragma unroll
        for (int c = 0; c < NJ; ++c) acc[a][c] = 0.f;
    float vsum = 0.f;

    // software pipeline over the slices: raw keys and v of the next slice are in flight while this one is evaluated
    float kx[NJ], vx = vx0;
#pragma unroll
    for (int c = 0; c < NJ; ++c) kx[c] = kx0[c];
    for (int h0 = 0; h0 < H; h0 += 64) {
        const float vh = vx;
        const bool hv = h0 + lane < H;
        bool kbig = false;
        float fk[NJ];                     // 2 log2e k of this slice; turned into exp(2k) on the factor path
#pragma unroll
        for (int c = 0; c < NJ; ++c) {
            const float x = hv ? kx[c] : 0.f;
            kbig |= fabsf(x) > kFactorLimit;
            fk[c] = kTwoLog2e * x;
        }
        if (h0 + 64 < H) {
            const int hn = h0 + 64 + lane;
            const int hc = hn < H ? hn : H - 1;
#pragma unroll
            for (int c = 0; c < NJ; ++c) kx[c] = ld(krow0, (size_t)c * H + hc);
            vx = hn < H ? ld(v, hc) : 0.f;
        }
        vsum += vh;
        const bool exact = qbig || __any(kbig);
        if (!exact) {
#pragma unroll
            for (int c = 0; c < NJ; ++c) fk[c] = fast_exp2(fk[c]);
#pragma unroll
            for (int a = 0; a < FW_R; ++a) {
                if (a < ni) {
                    const float eq = s_e[a * Hp + h0 + lane];
#pragma unroll
                    for (int c = 0; c < NJ; ++c) acc[a][c] = __builtin_fmaf(vh, r_from_factors(eq, fk[c]), acc[a][c]);
                }
            }
        } else {
#pragma unroll
            for (int a = 0; a < FW_R; ++a) {
                if (a < ni) {
                    const float sq = s_s[a * Hp + h0 + lane];
#pragma unroll
                    for (int c = 0; c < NJ; ++c) acc[a][c] = __builtin_fmaf(vh, r_from_sum(sq, fk[c]), acc[a][c]);
                }
            }
        }
    }
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
        if (a < ni) s_S[a * spitch + jcol0 + c] = tot;
    }
}

template <typename T>
__global__ __launch_bounds__(FW_THREADS, 3) void k_fwd_fused(
    const T *__restrict__ Qp, const T *__restrict__ Kp, const T *__restrict__ V, const T *__restrict__ v,
    const int *__restrict__ key_len, float *__restrict__ C, float *__restrict__ P,
    int B, int Tq, int Tk, int H, int Dv, int tiles, int Hp, int spitch, int sorted) {
    extern __shared__ float smem[];
    float *s_e = smem;                       // [FW_R][Hp]  exp(2q)
    float *s_s = s_e + FW_R * Hp;            // [FW_R][Hp]  2 log2e q
    float *s_S = s_s + FW_R * Hp;            // [FW_R][spitch]  scores, then probabilities
    __shared__ int s_b;

    const int lane = lane_id(), w = wave_id();

    // ---- which (sample, row tile): XCD x takes the samples of rank x, x+8, ... (rank 0 = most valid keys)
    const int xcd = blockIdx.x % FW_XCD, idx = blockIdx.x / FW_XCD;
    const int rank = xcd + FW_XCD * (idx / tiles), tile = idx % tiles;
    if (rank >= B) return;
    int b = rank;
    if (sorted) {
        // rank of a sample = how many samples come before it when ordered by valid keys, most first
        int *s_len = reinterpret_cast<int *>(smem);            // B ints; the staging below reuses the space
        for (int o = threadIdx.x; o < B; o += FW_THREADS) s_len[o] = clamp_len(key_len[o], Tk);
        __syncthreads();
        for (int cand = threadIdx.x; cand < B; cand += FW_THREADS) {
            const int lc = s_len[cand];
            int r = 0;
            for (int o = 0; o < B; ++o) {
                const int lo = s_len[o];
                r += (lo > lc) || (lo == lc && o < cand);
            }
            if (r == rank) s_b = cand;
        }
        __syncthreads();
        b = s_b;
    }
    const int L = clamp_len(key_len[b], Tk);
    const int r0 = (int)(((long long)Tq * tile) / tiles), r1 = (int)(((long long)Tq * (tile + 1)) / tiles);
    const int ni = r1 - r0;                                   // 1..FW_R

    float *Pb = P + ((size_t)b * Tq + r0) * Tk;
    float *Cb = C + ((size_t)b * Tq + r0) * Dv;
    if (L == 0) {                                             // no valid key: zeros
        for (int e = threadIdx.x; e < ni * Tk; e += FW_THREADS) Pb[e] = 0.f;
        for (int e = threadIdx.x; e < ni * Dv; e += FW_THREADS) Cb[e] = 0.f;
        return;
    }

    const T *kb = Kp + (size_t)b * Tk * H;
    const int n_chunk = (L + FW_W * FW_RJ - 1) / (FW_W * FW_RJ);
    // first slice of this wave's keys of chunk `ch` (rows past its run are clamped; they are not used)
    float kx0[FW_RJ], vx0;
    auto prefetch = [&](int ch, int &j_lo, int &nj) {
        const int c_lo = (int)(((long long)L * ch) / n_chunk), c_hi = (int)(((long long)L * (ch + 1)) / n_chunk);
        const int nk = c_hi - c_lo;                            // <= FW_W * FW_RJ
        j_lo = c_lo + (nk * w) / FW_W;
        nj = c_lo + (nk * (w + 1)) / FW_W - j_lo;              // 0..FW_RJ
        const int hc = lane < H ? lane : H - 1;
#pragma unroll
        for (int c = 0; c < FW_RJ; ++c) {
            const int j = min(j_lo + c, L - 1);
            kx0[c] = ld(kb, (size_t)j * H + hc);
        }
        vx0 = lane < H ? ld(v, hc) : 0.f;
    };
    int j_lo, nj;
    prefetch(0, j_lo, nj);

    // ---- A: stage the query rows
    const T *qb = Qp + ((size_t)b * Tq + r0) * H;
    bool big = false;
    constexpr int QB = 8;                       // loads in flight per thread
    for (int base = 0; base < FW_R * Hp; base += QB * FW_THREADS) {
        float x[QB];
        bool ok[QB];
#pragma unroll
        for (int u = 0; u < QB; ++u) {
            const int e = base + u * FW_THREADS + threadIdx.x;
            const int a = e / Hp, h = e - a * Hp;
            ok[u] = a < ni && h < H;
            x[u] = ok[u] ? ld(qb, (size_t)a * H + h) : 0.f;
        }
#pragma unroll
        for (int u = 0; u < QB; ++u) {
            const int e = base + u * FW_THREADS + threadIdx.x;
            if (e < FW_R * Hp) {
                big |= fabsf(x[u]) > kFactorLimit;
                const float sc = kTwoLog2e * x[u];
                s_s[e] = sc;
                s_e[e] = ok[u] ? fast_exp2(sc) : 0.f;
            }
        }
    }
    const bool qbig = __syncthreads_or(big) != 0;

    // ---- B: scores, keys in chunks of at most FW_W * FW_RJ
    for (int ch = 0; ch < n_chunk; ++ch) {
        if (ch > 0) prefetch(ch, j_lo, nj);
        const T *krow0 = kb + (size_t)j_lo * H;
#define FW_CASE(N) \
    case N: fw_score_wave<T, N>(s_e, s_s, Hp, ni, qbig, krow0, H, v, s_S, spitch, j_lo, kx0, vx0); break;
        switch (nj) {
            FW_CASE(1) FW_CASE(2) FW_CASE(3) FW_CASE(4) FW_CASE(5) FW_CASE(6) FW_CASE(7) FW_CASE(8)
            default: break;
        }
#undef FW_CASE
    }
    __syncthreads();

    // ---- C: softmax, wave r <-> row r; probabilities replace the scores in LDS
    const int Lp = (L + 3) & ~3;
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

    // ---- D: context rows = P V.  Lane l owns column n0 + l; per key one V row load feeds two 4-row MFMAs.
    const T *vb = V + (size_t)b * Tk * Dv;
    const int lr = lane & 3;
    for (int n0 = w * 64; n0 < Dv; n0 += FW_W * 64) {
        const int n = n0 + lane;
        const bool nv = n < Dv;
        const int nc = nv ? n : Dv - 1;
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 2
        for (int k0 = 0; k0 < Lp; k0 += 4) {
            const float4 pa = *reinterpret_cast<const float4 *>(s_S + lr * spitch + k0);
            const float4 pb = *reinterpret_cast<const float4 *>(s_S + (4 + lr) * spitch + k0);
            float vv[4];
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)      // keys past L carry P = 0; read the last valid row instead
                vv[kk] = ld(vb, (size_t)min(k0 + kk, L - 1) * Dv + nc);
            acc0 = __builtin_amdgcn_mfma_f32_4x4x1f32(pa.x, vv[0], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_4x4x1f32(pb.x, vv[0], acc1, 0, 0, 0);
            acc0 = __builtin_amdgcn_mfma_f32_4x4x1f32(pa.y, vv[1], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_4x4x1f32(pb.y, vv[1], acc1, 0, 0, 0);
            acc0 = __builtin_amdgcn_mfma_f32_4x4x1f32(pa.z, vv[2], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_4x4x1f32(pb.z, vv[2], acc1, 0, 0, 0);
            acc0 = __builtin_amdgcn_mfma_f32_4x4x1f32(pa.w, vv[3], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_4x4x1f32(pb.w, vv[3], acc1, 0, 0, 0);
        }
        if (nv) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (r < ni) Cb[(size_t)r * Dv + n] = acc0[r];
                if (4 + r < ni) Cb[(size_t)(4 + r) * Dv + n] = acc1[r];
            }
        }
    }
}

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
    const int ranks_per_xcd = (s.B + FW_XCD - 1) / FW_XCD;
    const int grid = FW_XCD * ranks_per_xcd * tiles;
    const int sorted = s.B <= 2048 ? 1 : 0;     // the in-kernel ranking is quadratic in B
    k_fwd_fused<T><<<grid, FW_THREADS, lds, st>>>((const T *)Qp, (const T *)Kp, (const T *)V, (const T *)v, key_len, C,
                                                  P, s.B, s.Tq, s.Tk, s.H, s.Dv, tiles, Hp, spitch, sorted);
    return hipGetLastError();
}

hipError_t launch_fwd_fused(const AttnShape &s, const void *Qp, const void *Kp, const void *V, const void *v,
                            const int *key_len, float *C, float *P, hipStream_t st) {
    return s.bf16 ? launch_fwd_fused_t<bf16_t>(s, Qp, Kp, V, v, key_len, C, P, st)
                  : launch_fwd_fused_t<float>(s, Qp, Kp, V, v, key_len, C, P, st);
}

}  // namespace echo
