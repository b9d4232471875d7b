// F1: attention scores  S[b,i,j] = sum_h v[h] * tanh(Qp[b,i,h] + Kp[b,j,h]),  j < L_b
// (scoring function: Section 4.1 broadcast add + tanh; Section 2, step 1).
//
// Lanes run along h, so every global and LDS access is contiguous.  A block
// owns a (rows x keys) tile of one sample; the exponentials exp(2q), exp(2k)
// of its rows are taken once while staging them into LDS, and each wave then
// evaluates an RI x RJ register tile of (i, j) pairs per 64-wide slice of h:
// one multiply-add, one reciprocal and one multiply-add per tanh.  The sum
// over h stays in registers (one partial per lane and pair) until the end,
// where a transposing butterfly leaves the total of pair p in lane p.
//
// STASH additionally writes tanh itself to a [B,Tq,Tk,H] map: the baseline
// that keeps the feature map, built for comparison only.
#include "common.hpp"
#include "kernels.hpp"

namespace echo {

constexpr int SC_RI = 8, SC_RJ = 8;        // register tile of one wave
constexpr int SC_WI = 2, SC_WJ = 2;        // waves per block along i and j
constexpr int SC_HC = 256;                 // h staged per pass
constexpr int SC_THREADS = 64 * SC_WI * SC_WJ;

template <typename T, bool STASH>
__global__ __launch_bounds__(SC_THREADS) void k_score(
    const T *__restrict__ Qp, const T *__restrict__ Kp, const T *__restrict__ v,
    const int *__restrict__ key_len, float *__restrict__ S, float *__restrict__ tmap,
    int Tq, int Tk, int H, int rows_per_blk, int n_jblk_max) {
    __shared__ float s_q[SC_WI * SC_RI][SC_HC];
    __shared__ float s_k[SC_WJ * SC_RJ][SC_HC];
    __shared__ int s_exact;

    const int b = blockIdx.z;
    const int L = clamp_len(key_len[b], Tk);
    // keys of this sample are cut into equal blocks of at most WJ*RJ
    const int n_jblk = (L + SC_WJ * SC_RJ - 1) / (SC_WJ * SC_RJ);
    if ((int)blockIdx.x >= n_jblk) return;
    const int keys_per_blk = (L + n_jblk - 1) / n_jblk;
    const int j_blk0 = blockIdx.x * keys_per_blk;
    const int nkeys = min(keys_per_blk, L - j_blk0);
    const int i_blk0 = blockIdx.y * rows_per_blk;
    const int nrows = min(rows_per_blk, Tq - i_blk0);
    (void)n_jblk_max;

    const int lane = lane_id(), w = wave_id();
    const int wi = w / SC_WJ, wj = w % SC_WJ;
    // rows / keys of this wave inside the block tile (even split)
    const int r_lo = (nrows * wi) / SC_WI, r_hi = (nrows * (wi + 1)) / SC_WI;
    const int c_lo = (nkeys * wj) / SC_WJ, c_hi = (nkeys * (wj + 1)) / SC_WJ;
    const int ni = r_hi - r_lo, nj = c_hi - c_lo;

    float acc[SC_RI][SC_RJ];
#pragma unroll
    for (int a = 0; a < SC_RI; ++a)
#pragma unroll
        for (int c = 0; c < SC_RJ; ++c) acc[a][c] = 0.f;
    float vsum = 0.f;

    const T *qb = Qp + (size_t)b * Tq * H;
    const T *kb = Kp + (size_t)b * Tk * H;

    for (int h0 = 0; h0 < H; h0 += SC_HC) {
        if (threadIdx.x == 0) s_exact = 0;
        __syncthreads();
        // ---- stage exp(2x) of the block's rows for this slice of h
        bool big = false;
        for (int idx = threadIdx.x; idx < (SC_WI * SC_RI + SC_WJ * SC_RJ) * SC_HC; idx += SC_THREADS) {
            const int row = idx / SC_HC, hh = idx % SC_HC, h = h0 + hh;
            float x = 0.f;
            bool ok;
            if (row < SC_WI * SC_RI) {
                // LDS row r of wave wi' holds tile row  split(wi') + (r % RI)
                const int wi2 = row / SC_RI, rr = row % SC_RI;
                const int lo = (nrows * wi2) / SC_WI, hi = (nrows * (wi2 + 1)) / SC_WI;
                ok = (lo + rr < hi) && h < H;
                if (ok) x = ld(qb, (size_t)(i_blk0 + lo + rr) * H + h);
                big |= fabsf(x) > kFactorLimit;
                s_q[row][hh] = ok ? fast_exp2(kTwoLog2e * x) : 0.f;
            } else {
                const int r2 = row - SC_WI * SC_RI;
                const int wj2 = r2 / SC_RJ, rr = r2 % SC_RJ;
                const int lo = (nkeys * wj2) / SC_WJ, hi = (nkeys * (wj2 + 1)) / SC_WJ;
                ok = (lo + rr < hi) && h < H;
                if (ok) x = ld(kb, (size_t)(j_blk0 + lo + rr) * H + h);
                big |= fabsf(x) > kFactorLimit;
                s_k[r2][hh] = ok ? fast_exp2(kTwoLog2e * x) : 0.f;
            }
        }
        if (big) s_exact = 1;
        __syncthreads();
        const bool exact = s_exact != 0;

        const int nslice = min(SC_HC, H - h0);
        for (int c0 = 0; c0 < nslice; c0 += 64) {
            const int h = h0 + c0 + lane;
            const bool hv = h < H;
            const float vh = hv ? ld(v, h) : 0.f;
            vsum += vh;
            if (!exact && !STASH) {
                float eq[SC_RI], ek[SC_RJ];
#pragma unroll
                for (int a = 0; a < SC_RI; ++a) eq[a] = s_q[wi * SC_RI + a][c0 + lane];
#pragma unroll
                for (int c = 0; c < SC_RJ; ++c) ek[c] = s_k[wj * SC_RJ + c][c0 + lane];
#pragma unroll
                for (int a = 0; a < SC_RI; ++a) {
                    if (a < ni) {
#pragma unroll
                        for (int c = 0; c < SC_RJ; ++c)
                            acc[a][c] = __builtin_fmaf(vh, r_from_factors(eq[a], ek[c]), acc[a][c]);
                    }
                }
            } else {
                // exact path: exponentiate the sum (rows with |x| beyond the factor limit), also used when stashing
                const int hc = hv ? h : 0;
#pragma unroll
                for (int a = 0; a < SC_RI; ++a) {
                    if (a < ni) {
                        const size_t irow = (size_t)(i_blk0 + r_lo + a);
                        const float sq = kTwoLog2e * ld(qb, irow * H + hc);
#pragma unroll
                        for (int c = 0; c < SC_RJ; ++c) {
                            if (c < nj) {
                                const size_t jrow = (size_t)(j_blk0 + c_lo + c);
                                const float sk = kTwoLog2e * ld(kb, jrow * H + hc);
                                const float r = r_from_sum(sq, sk);
                                acc[a][c] = __builtin_fmaf(vh, r, acc[a][c]);
                                if (STASH && hv)
                                    tmap[(((size_t)b * Tq + irow) * Tk + jrow) * H + h] = __builtin_fmaf(-2.f, r, 1.f);
                            }
                        }
                    }
                }
            }
        }
        __syncthreads();
    }

    // S = sum_h v (1 - 2r) = sum_h v - 2 sum_h v r ; per lane first, then across lanes
    float flat[SC_RI * SC_RJ];
#pragma unroll
    for (int a = 0; a < SC_RI; ++a)
#pragma unroll
        for (int c = 0; c < SC_RJ; ++c) flat[a * SC_RJ + c] = __builtin_fmaf(-2.f, acc[a][c], vsum);
    const float tot = wave_transpose_sum<SC_RI * SC_RJ>(flat);
    const int a = lane / SC_RJ, c = lane % SC_RJ;
    if (a < ni && c < nj)
        S[((size_t)b * Tq + i_blk0 + r_lo + a) * Tk + j_blk0 + c_lo + c] = tot;
}

template <typename T, bool STASH>
static hipError_t launch_score_t(const AttnShape &s, const void *Qp, const void *Kp, const void *v,
                                 const int *key_len, float *S, float *tmap, hipStream_t st) {
    const int max_rows = SC_WI * SC_RI;
    const int n_iblk = (s.Tq + max_rows - 1) / max_rows;
    const int rows_per_blk = (s.Tq + n_iblk - 1) / n_iblk;
    const int n_jblk = (s.Tk + SC_WJ * SC_RJ - 1) / (SC_WJ * SC_RJ);
    dim3 grid(n_jblk, n_iblk, s.B);
    k_score<T, STASH><<<grid, SC_THREADS, 0, st>>>((const T *)Qp, (const T *)Kp, (const T *)v, key_len, S, tmap,
                                                   s.Tq, s.Tk, s.H, rows_per_blk, n_jblk);
    return hipGetLastError();
}

hipError_t launch_score(const AttnShape &s, const void *Qp, const void *Kp, const void *v, const int *key_len,
                        float *S, float *tmap, hipStream_t st) {
    if (s.bf16) {
        return tmap ? launch_score_t<bf16_t, true>(s, Qp, Kp, v, key_len, S, tmap, st)
                    : launch_score_t<bf16_t, false>(s, Qp, Kp, v, key_len, S, tmap, st);
    }
    return tmap ? launch_score_t<float, true>(s, Qp, Kp, v, key_len, S, tmap, st)
                : launch_score_t<float, false>(s, Qp, Kp, v, key_len, S, tmap, st);
}

}  // namespace echo
