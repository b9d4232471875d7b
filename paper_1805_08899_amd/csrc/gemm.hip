// The dense contractions of the layer on the matrix cores, fp32 in and out
// (v_mfma_f32_16x16x4_f32):
//   F3  context[b] = P[b] . V[b]                 (Section 2, step 2)
//   B1  dV[b] = P[b]^T . dC[b],  dP[b] = dC[b] . V[b]^T   (Eq. 2: only inputs needed)
//   B2  dS = P (dP - rowsum(P dP)), fused behind dP so dP never leaves the CU
//
// Operand layout of one 16x16x4 step, lane l:  A[m = l%16][k = l/16],
// B[k = l/16][n = l%16], D[m = 4*(l/16) + r][n = l%16] in accumulator r.
#include "common.hpp"
#include "kernels.hpp"

namespace echo {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float comp4(const float4 &x, int c) { return c == 0 ? x.x : c == 1 ? x.y : c == 2 ? x.z : x.w; }
__device__ __forceinline__ f32x4 mfma16(float a, float b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// ---------------------------------------------------------------------------
// out[b, m, n] = sum_k A(m, k) * Bm[b, k, n]
//   TRANS_A = false: A(m, k) = P[b, m, k]   M = Tq, K = L_b   (context)
//   TRANS_A = true : A(m, k) = P[b, k, m]   M = Tk, K = Tq    (dV; rows m >= L_b are zero)
// A wave owns 16 rows x 64 columns: each lane loads four consecutive columns
// of Bm (one 16-byte load) and feeds component c to column tile c, so the
// output columns of tile c are n0 + 4*(l%16) + c and the store is 16 bytes too.
// N must be a multiple of 4.
template <typename TB, bool TRANS_A>
__device__ __forceinline__ void pv_block(const float *__restrict__ P, const TB *__restrict__ Bm,
                                         const int *__restrict__ key_len, float *__restrict__ out,
                                         int Tq, int Tk, int N, int b, int by, int bx, int acc_out) {
    const int L = clamp_len(key_len[b], Tk);
    const int lane = lane_id(), w = wave_id();
    const int M = TRANS_A ? Tk : Tq;
    const int K = TRANS_A ? Tq : L;
    const int Mvalid = TRANS_A ? L : Tq;      // rows that can be non-zero
    const int m0 = by * 16;
    const int n0 = (bx * 4 + w) * 64;
    if (n0 >= N) return;
    const int lm = lane & 15, lk = lane >> 4;
    const int ncol = n0 + 4 * lm;             // first of this lane's four columns
    const bool nok = ncol < N;
    const float *Pb = P + (size_t)b * Tq * Tk;
    const TB *Bb = Bm + (size_t)b * (TRANS_A ? Tq : Tk) * N;

    f32x4 acc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] = (f32x4){0.f, 0.f, 0.f, 0.f};

    if (m0 < Mvalid) {
        const int m = m0 + lm;
        constexpr int U = TRANS_A ? 16 : 8;       // k-steps whose loads are in flight together
        for (int kb0 = 0; kb0 < K; kb0 += 4 * U) {
            float a[U];
            float4 bv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = kb0 + 4 * u + lk;
                a[u] = 0.f;
                bv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (kb0 + 4 * u < K) {            // uniform
                    if (m < Mvalid && k < K) a[u] = TRANS_A ? Pb[(size_t)k * Tk + m] : Pb[(size_t)m * Tk + k];
                    if (k < K && nok) bv[u] = ld4(Bb, (size_t)k * N + ncol);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (kb0 + 4 * u < K) {
                    acc[0] = mfma16(a[u], bv[u].x, acc[0]);
                    acc[1] = mfma16(a[u], bv[u].y, acc[1]);
                    acc[2] = mfma16(a[u], bv[u].z, acc[2]);
                    acc[3] = mfma16(a[u], bv[u].w, acc[3]);
                }
            }
        }
    }
    if (!nok) return;
    float *ob = out + (size_t)b * M * N;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int m = m0 + 4 * lk + r;
        if (m < M) {
            float4 o = make_float4(acc[0][r], acc[1][r], acc[2][r], acc[3][r]);
            float4 *dst = reinterpret_cast<float4 *>(ob + (size_t)m * N + ncol);
            if (acc_out) {                       // add to what the earlier decoder steps left
                const float4 old = *dst;
                o.x += old.x;
                o.y += old.y;
                o.z += old.z;
                o.w += old.w;
            }
            store4_streaming(ob + (size_t)m * N + ncol, o);
        }
    }
}

template <typename TB, bool TRANS_A>
__global__ __launch_bounds__(256) void k_pv(const float *__restrict__ P, const TB *__restrict__ Bm,
                                            const int *__restrict__ key_len, float *__restrict__ out,
                                            int Tq, int Tk, int N) {
    pv_block<TB, TRANS_A>(P, Bm, key_len, out, Tq, Tk, N, blockIdx.z, blockIdx.y, blockIdx.x, 0);
}

hipError_t launch_context(const AttnShape &s, const float *P, const void *V, const int *key_len, float *C,
                          hipStream_t st) {
    dim3 grid((s.Dv + 255) / 256, (s.Tq + 15) / 16, s.B);
    if (s.bf16)
        k_pv<bf16_t, false><<<grid, 256, 0, st>>>(P, (const bf16_t *)V, key_len, C, s.Tq, s.Tk, s.Dv);
    else
        k_pv<float, false><<<grid, 256, 0, st>>>(P, (const float *)V, key_len, C, s.Tq, s.Tk, s.Dv);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// dS for (b, 16 query rows).  Waves take key tiles of 16 in turn and compute
// dP[i, j] = sum_d dC[i, d] V[j, d] into LDS; then each wave finishes four
// rows: r = sum_j P dP, dS = P (dP - r).  dS rows have pitch `pitch` floats and
// are zero at j >= L_b (pads included).  Dv must be a multiple of 4.
// A lane loads four consecutive d of its row for both operands and spends
// them on four MFMA steps, so the k index of step c is d0 + 4*(l/16) + c on
// both sides.
template <typename TV, int G, int RB>
__device__ __forceinline__ void dscore_block(const float *__restrict__ dC, const TV *__restrict__ V,
                                             const float *__restrict__ P, const int *__restrict__ key_len,
                                             float *__restrict__ dS, float *__restrict__ ds_rowsum,
                                             float *__restrict__ s_dp, int b, int i0, int Tq, int Tk, int Dv,
                                             int pitch) {
    const int L = clamp_len(key_len[b], Tk);
    const int lane = lane_id(), w = wave_id();
    const int lm = lane & 15, lk = lane >> 4;
    const int pitch16 = (Tk + 15) / 16 * 16 + 4;
    const float *dCb = dC + (size_t)b * Tq * Dv;
    const TV *Vb = V + (size_t)b * Tk * Dv;

    // Wave w takes key tiles w, w+4, ..., G at a time so that one fragment of dC feeds G products (the
    // kernel is bound by what the L2 can deliver, not by the matrix cores); tiles past the sample's last one are
    // neither loaded nor multiplied.  RB = 2: the block owns 32 query rows, two fragments of dC, so that every
    // V fragment feeds two products and the sample's V rows pass through half as many blocks.  The sum over d runs
    // in stages of U 16-wide slices; the loads of the next stage are in flight while the current one is multiplied.
    // Rows and keys past the end are clamped for loading; what they produce is never read.  Columns past Dv are zeroed.
    const int n_jt = (L + 15) / 16;
    constexpr int U = RB == 2 ? 1 : 2;
    const int n_st = (Dv + 16 * U - 1) / (16 * U);            // stages
    const bool ragged = Dv % (16 * U) != 0;
    const float *dCrow[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) dCrow[rb] = dCb + (size_t)min(i0 + 16 * rb + lm, Tq - 1) * Dv;
    for (int jt0 = w; jt0 < n_jt; jt0 += 4 * G) {              // this wave's tiles jt0, jt0 + 4, jt0 + 8, ...
        const TV *vrow[G];
#pragma unroll
        for (int k = 0; k < G; ++k) vrow[k] = Vb + (size_t)min((jt0 + 4 * k) * 16 + lm, Tk - 1) * Dv;
        float4 a[RB][U], bv[G][U], an[RB][U], bn[G][U];
#pragma unroll
        for (int k = 0; k < G; ++k)
#pragma unroll
            for (int u = 0; u < U; ++u) bv[k][u] = bn[k][u] = make_float4(0.f, 0.f, 0.f, 0.f);
        // key tiles of this group that exist (the same in all lanes): the others are neither loaded nor multiplied
        bool live[G];
#pragma unroll
        for (int k = 0; k < G; ++k) live[k] = jt0 + 4 * k < n_jt;
        auto load = [&](float4 (&da)[RB][U], float4 (&db)[G][U], int st) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int d = min((st * U + u) * 16 + 4 * lk, Dv - 4);
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) da[rb][u] = ld4(dCrow[rb], (size_t)d);
#pragma unroll
                for (int k = 0; k < G; ++k)
                    if (live[k]) db[k][u] = ld4(vrow[k], (size_t)d);
            }
        };
        load(a, bv, 0);
        f32x4 acc[RB][G];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int k = 0; k < G; ++k) acc[rb][k] = (f32x4){0.f, 0.f, 0.f, 0.f};
        for (int st = 0; st < n_st; ++st) {
            load(an, bn, min(st + 1, n_st - 1));
            if (ragged && st == n_st - 1) {                      // columns past Dv add nothing
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if ((st * U + u) * 16 + 4 * lk >= Dv) {
#pragma unroll
                        for (int rb = 0; rb < RB; ++rb) a[rb][u] = make_float4(0.f, 0.f, 0.f, 0.f);
                    }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
                    for (int k = 0; k < G; ++k) if (live[k]) acc[rb][k] = mfma16(a[rb][u].x, bv[k][u].x, acc[rb][k]);
                }
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
                    for (int k = 0; k < G; ++k) if (live[k]) acc[rb][k] = mfma16(a[rb][u].y, bv[k][u].y, acc[rb][k]);
                }
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
                    for (int k = 0; k < G; ++k) if (live[k]) acc[rb][k] = mfma16(a[rb][u].z, bv[k][u].z, acc[rb][k]);
                }
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
#pragma unroll
                    for (int k = 0; k < G; ++k) if (live[k]) acc[rb][k] = mfma16(a[rb][u].w, bv[k][u].w, acc[rb][k]);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) a[rb][u] = an[rb][u];
#pragma unroll
                for (int k = 0; k < G; ++k) bv[k][u] = bn[k][u];
            }
        }
#pragma unroll
        for (int k = 0; k < G; ++k) {
            const int jt = jt0 + 4 * k;
            if (jt < n_jt) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) s_dp[(16 * rb + 4 * lk + r) * pitch16 + jt * 16 + lm] = acc[rb][k][r];
            }
        }
    }
    // P of the rows this wave finishes (w, w + 4, ...), the first NP keys per lane of each: requested together
    // before the barrier (the registers of the product loop are free by now), where loading row after row inside
    // the loop below put one trip to memory behind the other
    constexpr int NP = 5, NR = 4 * RB;
    float pr[NR][NP];
#pragma unroll
    for (int t = 0; t < NR; ++t) {
        const float *p = P + ((size_t)b * Tq + min(i0 + w + 4 * t, Tq - 1)) * Tk;
#pragma unroll
        for (int c = 0; c < NP; ++c) pr[t][c] = p[min(lane + 64 * c, Tk - 1)];
    }
    lds_barrier();

#pragma unroll
    for (int t = 0; t < NR; ++t) {
        const int rr = w + 4 * t, i = i0 + rr;
        if (i < Tq) {
            const float *p = P + ((size_t)b * Tq + i) * Tk;
            const float *dp = s_dp + rr * pitch16;
            float *ds = dS + ((size_t)b * Tq + i) * pitch;
            float r = 0.f;
#pragma unroll
            for (int c = 0; c < NP; ++c)
                if (lane + 64 * c < L) r += pr[t][c] * dp[lane + 64 * c];
            for (int j = lane + 64 * NP; j < L; j += 64) r += p[j] * dp[j];
            r = wave_sum(r);
            float tot = 0.f;
#pragma unroll
            for (int c = 0; c < NP; ++c) {
                const int j = lane + 64 * c;
                if (j < pitch) {
                    float x = 0.f;
                    if (j < L) x = pr[t][c] * (dp[j] - r);
                    ds[j] = x;
                    tot += x;
                }
            }
            for (int j = lane + 64 * NP; j < pitch; j += 64) {
                float x = 0.f;
                if (j < L) x = p[j] * (dp[j] - r);
                ds[j] = x;
                tot += x;
            }
            tot = wave_sum(tot);
            if (lane == 0) ds_rowsum[(size_t)b * Tq + i] = tot;
        }
    }
}


// The same for short key axes (Tk <= kDsplitMaxTk): latency, not arithmetic, decides here, so the four waves
// split d instead of the key tiles.  Wave w owns the columns d of every fourth 128-wide chunk, keeps its slice
// of the 16 dC rows in registers across the key tiles when Dv <= 512, has the V slice of the next key tile in
// flight while the current one is multiplied, and leaves a partial dP tile in its own LDS plane; the planes
// are added in wave order by the finishing phase, whose P rows were requested at the very start.
// Rows and keys past the end are clamped for loading; what they produce is never read.
constexpr int kDsplitMaxTk = 128;
constexpr int kDs32MaxTk = 384;      // 32 rows x (Tk + 4) floats: 48.5 KB of LDS at most, three blocks per CU

// The finishing phase of a dS block for short key axes: the four waves' planes of partial dP are added in wave order,
// then dS = P (dP - sum_j P dP) for rows w, w+4, w+8, w+12 of the tile (pr: their P, two keys per lane).
__device__ __forceinline__ void dsplit_finish(const float (&pr)[4][2], const float *__restrict__ s_dp,
                                              float *__restrict__ dS, float *__restrict__ ds_rowsum, int b, int i0,
                                              int Tq, int L, int pitch, int pitch16, int plane) {
    const int lane = lane_id(), w = wave_id();

    // the four rows together: r = sum_j P dP and sum_j dS by transposing reductions (sum of row t ends up in
    // lanes 16 t .. 16 t + 15), so the exchanges of the rows overlap instead of queueing behind each other
    float dp[4][2], rsum[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int rr = w + 4 * t;
        rsum[t] = 0.f;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int j = lane + 64 * u;
            const float *q = s_dp + rr * pitch16 + min(j, pitch16 - 1);
            const float x = ((q[0] + q[plane]) + q[2 * plane]) + q[3 * plane];
            dp[t][u] = j < L ? x : 0.f;
            rsum[t] = __builtin_fmaf(j < L ? pr[t][u] : 0.f, dp[t][u], rsum[t]);
        }
    }
    const float r4 = wave_transpose_sum<4>(rsum);
    float tsum[4], dsv[4][2];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const float r = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(r4), 16 * t));
        tsum[t] = 0.f;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int j = lane + 64 * u;
            dsv[t][u] = j < L ? pr[t][u] * (dp[t][u] - r) : 0.f;
            tsum[t] += dsv[t][u];
        }
    }
    const float t4 = wave_transpose_sum<4>(tsum);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int i = i0 + w + 4 * t;
        if (i < Tq) {
            float *ds = dS + ((size_t)b * Tq + i) * pitch;
#pragma unroll
            for (int u = 0; u < 2; ++u)
                if (lane + 64 * u < pitch) store_streaming(&ds[lane + 64 * u], dsv[t][u]);
            if (lane == 16 * t) ds_rowsum[(size_t)b * Tq + i] = t4;
        }
    }
}

// The general form (any width of the value rows): two register groups of a whole round of V slices each, one in
// flight; with more than one round the dC slices are fetched per key tile and round.
template <typename TV>
__device__ __forceinline__ void dscore_block_dsplit(const float *__restrict__ dC, const TV *__restrict__ V,
                                                    const float *__restrict__ P, const int *__restrict__ key_len,
                                                    float *__restrict__ dS, float *__restrict__ ds_rowsum,
                                                    float *__restrict__ s_dp, int b, int i0, int Tq, int Tk,
                                                    int Dv, int pitch) {
    const int lane = lane_id(), w = wave_id();
    const int lm = lane & 15, lk = lane >> 4;
    const int pitch16 = (Tk + 15) / 16 * 16 + 4;
    const int plane = 16 * pitch16;
    // P of the rows this wave finishes (rows w, w+4, w+8, w+12 of the tile), two keys per lane
    float pr[4][2];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int i = min(i0 + w + 4 * t, Tq - 1);
#pragma unroll
        for (int u = 0; u < 2; ++u) pr[t][u] = P[((size_t)b * Tq + i) * Tk + min(lane + 64 * u, Tk - 1)];
    }
    const float *dCrow = dC + ((size_t)b * Tq + min(i0 + lm, Tq - 1)) * Dv;
    const TV *Vb = V + (size_t)b * Tk * Dv;
    constexpr int U = 8;                          // 16-wide slices of d per wave and round
    const int rounds = (Dv + 64 * U - 1) / (64 * U);
    float4 a[U], bcur[U], bnxt[U];
    auto load_a = [&](int r) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int d = (4 * r + w) * 16 * U + 16 * u + 4 * lk;
            const float4 x = ld4(dCrow, (size_t)min(d, Dv - 4));
            a[u] = d < Dv ? x : make_float4(0.f, 0.f, 0.f, 0.f);     // columns past Dv add nothing
        }
    };
    auto load_b = [&](float4 (&dst)[U], int it) {
        const int jt = it / rounds, r = it % rounds;
        const TV *row = Vb + (size_t)min(jt * 16 + lm, Tk - 1) * Dv;
#pragma unroll
        for (int u = 0; u < U; ++u) dst[u] = ld4(row, (size_t)min((4 * r + w) * 16 * U + 16 * u + 4 * lk, Dv - 4));
    };
    // the first slices do not depend on the sample's key count (key tile 0 always exists in memory): they
    // leave before key_len[b] has arrived
    load_b(bcur, 0);
    load_a(0);
    const int L = clamp_len(key_len[b], Tk);
    const int n_jt = (L + 15) / 16;
    const int items = n_jt * rounds;
    f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < items; ++it) {
        const int jt = it / rounds, r = it % rounds;
        load_b(bnxt, min(it + 1, items - 1));
        if (rounds > 1 && it > 0) load_a(r);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            acc = mfma16(a[u].x, bcur[u].x, acc);
            acc = mfma16(a[u].y, bcur[u].y, acc);
            acc = mfma16(a[u].z, bcur[u].z, acc);
            acc = mfma16(a[u].w, bcur[u].w, acc);
        }
        if (r == rounds - 1) {
#pragma unroll
            for (int q = 0; q < 4; ++q) s_dp[w * plane + (4 * lk + q) * pitch16 + jt * 16 + lm] = acc[q];
            acc = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int u = 0; u < U; ++u) bcur[u] = bnxt[u];
    }
    lds_barrier();
    dsplit_finish(pr, s_dp, dS, ds_rowsum, b, i0, Tq, L, pitch, pitch16, plane);
}

// Short key axes, value rows of at most 1024 columns, operands through LDS.  A quarter of a wave that reads the operand
// layout of the matrix cores straight from memory asks for the same 16 bytes of 16 different rows; with rows a
// multiple of 128 bytes apart these requests queue in the CU's L1 (measured: 37 KB/us per CU, against 90 to 110
// for loads of whole row pieces, and 67 with rows 2064 bytes apart).  Here a wave loads its 128 columns of 16 rows
// as 8 loads of two 512-byte row pieces each (lanes along d), writes them row by row into its own 16 x 132 floats
// of LDS and reads them back in operand layout (row l % 16, 16 bytes at column 16 u + 4 (l / 16): conflict-free at
// this pitch).  The region belongs to one wave, so no barrier is involved; the V slice of the next key tile is in
// flight in registers while the current one is multiplied.
// ROUNDS = 1 (up to 512 columns): the partial dP tiles stay in registers until the end and then go into the same
// region, which the finishing phase reads as the wave's plane.
// ROUNDS = 2 (513 to 1024 columns): the dC slices of both rounds stay in registers, the steps run over (key tile,
// round), and the partial dP tiles go to planes of their own behind the staging regions as each key tile finishes
// (there is no room to keep eight of them in registers next to two rounds of dC).  The general form above fetches
// the dC slices again for every key tile and round and waits for them each time.
constexpr int kStagePitch = 132;                 // floats; 16 rows of it are a wave's region
template <typename TV, int ROUNDS>
__device__ __forceinline__ void dscore_block_dsplit_lds(const float *__restrict__ dC, const TV *__restrict__ V,
                                                        const float *__restrict__ P, const int *__restrict__ key_len,
                                                        float *__restrict__ dS, float *__restrict__ ds_rowsum,
                                                        float *__restrict__ s_stage, int b, int i0, int Tq, int Tk,
                                                        int Dv, int pitch) {
    const int lane = lane_id(), w = wave_id();
    const int lm = lane & 15, lk = lane >> 4;
    const int pitch16 = (Tk + 15) / 16 * 16 + 4;
    constexpr int region = 16 * kStagePitch;
    constexpr int NT = ROUNDS == 1 ? kDsplitMaxTk / 16 : 1;       // dP tiles kept in registers
    // the planes of partial dP: the staging regions themselves (one round) or planes behind them
    float *planes = ROUNDS == 1 ? s_stage : s_stage + 4 * region;
    const int plane = ROUNDS == 1 ? region : 16 * pitch16;
    // P of the rows this wave finishes (rows w, w+4, w+8, w+12 of the tile), two keys per lane
    float pr[4][2];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int i = min(i0 + w + 4 * t, Tq - 1);
#pragma unroll
        for (int u = 0; u < 2; ++u) pr[t][u] = P[((size_t)b * Tq + i) * Tk + min(lane + 64 * u, Tk - 1)];
    }
    constexpr int U = 8;                          // 16-wide slices of d per wave and round
    float *st = s_stage + w * region;             // this wave's region
    const int cr = lane >> 5, cc = 4 * (lane & 31);               // loading: row of the pair, column in the chunk
    const float *dCb = dC + (size_t)b * Tq * Dv;
    const TV *Vb = V + (size_t)b * Tk * Dv;
    float4 a[ROUNDS][U], bcur[U], bnxt[U];
    auto col_of = [&](int r) { return min((4 * r + w) * 16 * U + cc, Dv - 4); };   // clamped for loading
    auto load_v = [&](float4 (&dst)[U], int it) {                 // step it = (key tile, round): 16 keys, two per load
        const int jt = it / ROUNDS, r = it % ROUNDS;
        const int col = col_of(r);
#pragma unroll
        for (int u = 0; u < U; ++u) dst[u] = ld4(Vb + (size_t)min(jt * 16 + 2 * u + cr, Tk - 1) * Dv, (size_t)col);
    };
    auto through_lds = [&](float4 (&dst)[U], const float4 (&src)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) *reinterpret_cast<float4 *>(st + (2 * u + cr) * kStagePitch + cc) = src[u];
#pragma unroll
        for (int u = 0; u < U; ++u) dst[u] = *reinterpret_cast<const float4 *>(st + lm * kStagePitch + 16 * u + 4 * lk);
    };
    // the first loads do not depend on the sample's key count (key tile 0 always exists in memory)
    load_v(bnxt, 0);
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
        const int col = col_of(r);
#pragma unroll
        for (int u = 0; u < U; ++u) a[r][u] = ld4(dCb + (size_t)min(i0 + 2 * u + cr, Tq - 1) * Dv, (size_t)col);
    }
    const int L = clamp_len(key_len[b], Tk);
    const int n_jt = (L + 15) / 16;
    const int items = n_jt * ROUNDS;
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
        through_lds(a[r], a[r]);
#pragma unroll
        for (int u = 0; u < U; ++u)                               // columns past Dv add nothing
            if ((4 * r + w) * 16 * U + 16 * u + 4 * lk >= Dv) a[r][u] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    through_lds(bcur, bnxt);
    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int jt = 0; jt < kDsplitMaxTk / 16; ++jt) {
        if (jt < n_jt) {                                           // uniform
#pragma unroll
            for (int r = 0; r < ROUNDS; ++r) {
                load_v(bnxt, min(jt * ROUNDS + r + 1, max(items - 1, 0)));
                f32x4 &d = acc[ROUNDS == 1 ? jt : 0];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    d = mfma16(a[r][u].x, bcur[u].x, d);
                    d = mfma16(a[r][u].y, bcur[u].y, d);
                    d = mfma16(a[r][u].z, bcur[u].z, d);
                    d = mfma16(a[r][u].w, bcur[u].w, d);
                }
                through_lds(bcur, bnxt);
            }
            if (ROUNDS > 1) {
#pragma unroll
                for (int q = 0; q < 4; ++q) planes[w * plane + (4 * lk + q) * pitch16 + jt * 16 + lm] = acc[0][q];
                acc[0] = (f32x4){0.f, 0.f, 0.f, 0.f};
            }
        }
    }
    if (ROUNDS == 1) {                            // the wave's plane of partial dP into its own region
#pragma unroll
        for (int jt = 0; jt < kDsplitMaxTk / 16; ++jt)
            if (jt < n_jt) {
#pragma unroll
                for (int q = 0; q < 4; ++q) st[(4 * lk + q) * pitch16 + jt * 16 + lm] = acc[ROUNDS == 1 ? jt : 0][q];
            }
    }
    lds_barrier();
    dsplit_finish(pr, planes, dS, ds_rowsum, b, i0, Tq, L, pitch, pitch16, plane);
}

// dV of one sample for a panel of 64 keys and 256 columns, 64 columns per wave: dV[j, n] = sum_i P[i, j] dC[i, n].
// Per step of four query rows a lane loads four consecutive keys of a P row and four consecutive columns of the dC
// row (16 bytes each) and spends them on 16 products: component ca of the keys with component cb of the columns,
// so product (ca, cb) holds keys m0 + 4 (row of the result tile) + ca and columns n0 + 4 (l % 16) + cb.  Two bytes
// of operands per lane and product, against five in the form with one key per lane (pv_block), which at the larger
// workloads was bound by what the L2 could deliver.  Needs Tk % 4 == 0 (16-byte loads of P rows).  Batches of U
// steps are double buffered.  Rows of masked keys (j >= L) come out as exact zeros whatever P holds there.
__device__ __forceinline__ void dv_tile64(const float *__restrict__ P, const float *__restrict__ dC,
                                          const int *__restrict__ key_len, float *__restrict__ dV, int Tq, int Tk,
                                          int Dv, int b, int by, int bx, int acc_out) {
    constexpr int U = 4;
    const int L = clamp_len(key_len[b], Tk);
    const int lane = lane_id(), w = wave_id();
    const int lm = lane & 15, lk = lane >> 4;
    const int m0 = by * 64, n0 = (bx * 4 + w) * 64;
    if (n0 >= Dv) return;
    const int kcol = m0 + 4 * lm;             // first of this lane's four keys
    const int ncol = n0 + 4 * lm;             // first of this lane's four columns
    const bool nok = ncol < Dv;
    const float *Pb = P + (size_t)b * Tq * Tk;
    const float *Cb = dC + (size_t)b * Tq * Dv;
    f32x4 acc[4][4];
#pragma unroll
    for (int ca = 0; ca < 4; ++ca)
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) acc[ca][cb] = (f32x4){0.f, 0.f, 0.f, 0.f};
    if (m0 < L) {
        const int kc = min(kcol, Tk - 4), nc = min(ncol, Dv - 4);       // clamped for loading
        float4 a[U], bv[U], an[U], bn[U];
        auto load = [&](float4 (&da)[U], float4 (&db)[U], int kb0) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int k = min(kb0 + 4 * u + lk, Tq - 1);
                da[u] = ld4(Pb, (size_t)k * Tk + kc);
                db[u] = ld4(Cb, (size_t)k * Dv + nc);
            }
        };
        load(a, bv, 0);
        for (int kb0 = 0; kb0 < Tq; kb0 += 4 * U) {
            load(an, bn, min(kb0 + 4 * U, Tq - 1));
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const bool row_on = kb0 + 4 * u + lk < Tq;               // rows past Tq add nothing
                float x[4];
#pragma unroll
                for (int ca = 0; ca < 4; ++ca) x[ca] = (row_on && kcol + ca < L) ? comp4(a[u], ca) : 0.f;
#pragma unroll
                for (int ca = 0; ca < 4; ++ca)
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb) acc[ca][cb] = mfma16(x[ca], comp4(bv[u], cb), acc[ca][cb]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                a[u] = an[u];
                bv[u] = bn[u];
            }
        }
    }
    if (!nok) return;
    float *ob = dV + (size_t)b * Tk * Dv;
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int ca = 0; ca < 4; ++ca) {
            const int m = m0 + 16 * lk + 4 * r + ca;
            if (m < Tk) {
                float4 o = make_float4(acc[ca][0][r], acc[ca][1][r], acc[ca][2][r], acc[ca][3][r]);
                if (acc_out) {                       // add to what the earlier decoder steps left
                    const float4 old = *reinterpret_cast<const float4 *>(ob + (size_t)m * Dv + ncol);
                    o.x += old.x;
                    o.y += old.y;
                    o.z += old.z;
                    o.w += old.w;
                }
                store4_streaming(ob + (size_t)m * Dv + ncol, o);
            }
        }
}

// dV of one sample for a 64-wide group of columns and ALL keys: dV[j, n0 .. n0+63] = sum_i P[i, j] dC[i, n0 ..].
// The block's slice of dC (Tq rows of 256 bytes) passes through the CU once; the earlier form, a block per 16 keys
// and 256 columns, read dC once per key tile and was bound by what the L2 could deliver at the larger workloads.
// Wave w owns key tiles w, w + 4, ... and works on KT of them at a time: per step of four query rows a lane loads
// KT values of P (one per key tile) and four consecutive columns of dC (one 16-byte load) and issues 4 KT products.
// Batches of U steps are double buffered: the loads of the next batch are in flight during the products of this one.
// Rows of masked keys (j >= L) come out as exact zeros.
template <int KT>
__device__ __forceinline__ void dv_cols_block(const float *__restrict__ P, const float *__restrict__ dC,
                                              const int *__restrict__ key_len, float *__restrict__ dV, int Tq, int Tk,
                                              int Dv, int b, int cg, int acc_out) {
    constexpr int U = KT == 1 ? 8 : KT == 2 ? 6 : KT == 3 ? 4 : 3;
    const int L = clamp_len(key_len[b], Tk);
    const int lane = lane_id(), w = wave_id();
    const int lm = lane & 15, lk = lane >> 4;
    const int ncol = cg * 64 + 4 * lm;
    const bool nok = ncol < Dv;
    const float *Pb = P + (size_t)b * Tq * Tk;
    const float *dCb = dC + (size_t)b * Tq * Dv + min(ncol, Dv - 4);
    float *dVb = dV + (size_t)b * Tk * Dv + ncol;
    const int n_kt = (Tk + 15) / 16;
    const int n_steps = (Tq + 3) / 4;
    for (int jt0 = w; jt0 < n_kt; jt0 += 4 * KT) {                 // this wave's tiles jt0, jt0 + 4, ...
        int m[KT];                                                  // key of this lane in tile t (clamped for loading)
#pragma unroll
        for (int t = 0; t < KT; ++t) m[t] = min((jt0 + 4 * t) * 16 + lm, Tk - 1);
        f32x4 acc[KT][4];
#pragma unroll
        for (int t = 0; t < KT; ++t)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[t][c] = (f32x4){0.f, 0.f, 0.f, 0.f};
        if (jt0 * 16 < L) {                                         // uniform: else all of the group's keys are masked
            float a[2][U][KT];
            float4 bv[2][U];
            auto load = [&](int buf, int st0) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int kc = min(4 * (st0 + u) + lk, Tq - 1);
#pragma unroll
                    for (int t = 0; t < KT; ++t) a[buf][u][t] = Pb[(size_t)kc * Tk + m[t]];
                    bv[buf][u] = ld4(dCb, (size_t)kc * Dv);
                }
            };
            auto mult = [&](int buf, int st0) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (st0 + u < n_steps) {                        // uniform
                        // query rows past Tq (last step only) were loaded from row Tq - 1: they add nothing.
                        // Masked here, at the point of use, so that nothing waits for the loads earlier.
                        const bool kv = 4 * (st0 + u) + lk < Tq;
#pragma unroll
                        for (int t = 0; t < KT; ++t) {
                            const float av = kv ? a[buf][u][t] : 0.f;
                            acc[t][0] = mfma16(av, bv[buf][u].x, acc[t][0]);
                            acc[t][1] = mfma16(av, bv[buf][u].y, acc[t][1]);
                            acc[t][2] = mfma16(av, bv[buf][u].z, acc[t][2]);
                            acc[t][3] = mfma16(av, bv[buf][u].w, acc[t][3]);
                        }
                    }
                }
            };
            load(0, 0);
            for (int st0 = 0; st0 < n_steps; st0 += 2 * U) {
                if (st0 + U < n_steps) load(1, st0 + U);
                mult(0, st0);
                if (st0 + 2 * U < n_steps) load(0, st0 + 2 * U);
                if (st0 + U < n_steps) mult(1, st0 + U);
            }
        }
        if (nok) {
#pragma unroll
            for (int t = 0; t < KT; ++t) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int j = (jt0 + 4 * t) * 16 + 4 * lk + r;
                    if (j < Tk) {
                        float4 o = make_float4(acc[t][0][r], acc[t][1][r], acc[t][2][r], acc[t][3][r]);
                        if (j >= L) o = make_float4(0.f, 0.f, 0.f, 0.f);      // masked key: its P column was not zeroed above
                        float *dst = dVb + (size_t)j * Dv;
                        if (acc_out) {                               // add to what the earlier decoder steps left
                            const float4 old = *reinterpret_cast<const float4 *>(dst);
                            o.x += old.x;
                            o.y += old.y;
                            o.z += old.z;
                            o.w += old.w;
                        }
                        store4_streaming(dst, o);
                    }
                }
            }
        }
    }
}

// For the recompute kernel: order[r] = b | L_b << 16 for the sample b with the
// r-th most valid keys (ties by index), or r-th in index order when `sorted` is 0.  With `fold` the second
// half runs lightest first: when the whole recompute grid is resident at once,
// blocks y and y + B/2 meet on one CU (two blocks per CU, placed in launch
// order), so heavy samples are paired with light ones.
__device__ __forceinline__ void rank_block(const int *__restrict__ key_len, int *__restrict__ order,
                                           int *__restrict__ s_len, int B, int Tk, int sorted, int fold) {
    if (sorted)
        for (int o = threadIdx.x; o < B; o += 256) s_len[o] = clamp_len(key_len[o], Tk);
    lds_barrier();
    const int half = (B + 1) / 2;
    for (int cand = threadIdx.x; cand < B; cand += 256) {
        int r = cand;
        const int lc = sorted ? s_len[cand] : clamp_len(key_len[cand], Tk);
        if (sorted) {
            r = 0;
            for (int o = 0; o < B; ++o) {
                const int lo = s_len[o];
                r += (lo > lc) || (lo == lc && o < cand);
            }
        }
        order[(fold && r >= half) ? half + (B - 1 - r) : r] = cand | (lc << 16);
    }
}

// Everything the backward pass needs before the recomputation, in one launch:
// blocks that produce dS (B1 + B2), blocks that produce dV (B1) and one block
// that ranks the samples.  The three kinds of block do not depend on each other.
template <typename TV, int KT>
__global__ __launch_bounds__(256, 3) void k_bwd_pre(const float *__restrict__ dC, const TV *__restrict__ V,
                                                 const float *__restrict__ P, const int *__restrict__ key_len,
                                                 float *__restrict__ dS, float *__restrict__ ds_rowsum,
                                                 int *__restrict__ order, float *__restrict__ dV, int B, int sorted,
                                                 int fold,
                                                 int Tq, int Tk, int Dv, int pitch, int s_tiles, int s_rows, int v_groups, int acc) {
    extern __shared__ float s_dp[];           // [s_rows][pitch16]; four planes of 16 rows when Tk <= kDsplitMaxTk
    __shared__ int s_len[kMaxSortedB];
    // The hardware deals blocks to the eight XCDs round-robin, so block id mod 8 names the XCD.  Sample b is
    // worked on by XCD b mod 8 only: its dC, V and P then pass through one L2 instead of eight.  Within an XCD the
    // long dS blocks of all its samples come first, then the dV blocks; the last block of the grid ranks.
    constexpr int kXcd = 8;
    const int spx = (B + kXcd - 1) / kXcd;                     // sample slots per XCD
    const int per_b = v_groups;                               // dV blocks per sample: one per 64 columns
    const int per_xcd = spx * (s_tiles + per_b);
    if ((int)blockIdx.x == kXcd * per_xcd) {
        rank_block(key_len, order, s_len, B, Tk, sorted, fold);
        return;
    }
    const int xcd = blockIdx.x % kXcd;
    int li = blockIdx.x / kXcd;
    if (li < spx * s_tiles) {
        const int b = xcd + kXcd * (li / s_tiles), i0 = (li % s_tiles) * s_rows;
        if (b >= B) return;
        if (Tk <= kDsplitMaxTk) {
            if (Dv <= 512) dscore_block_dsplit_lds<TV, 1>(dC, V, P, key_len, dS, ds_rowsum, s_dp, b, i0, Tq, Tk, Dv, pitch);
            else if (Dv <= 1024) dscore_block_dsplit_lds<TV, 2>(dC, V, P, key_len, dS, ds_rowsum, s_dp, b, i0, Tq, Tk, Dv, pitch);
            else dscore_block_dsplit<TV>(dC, V, P, key_len, dS, ds_rowsum, s_dp, b, i0, Tq, Tk, Dv, pitch);
        } else {
            // a wave's key tiles in groups of four, or of five where that takes all of them at once (17 to 20 key tiles)
            const bool five = (Tk + 15) / 16 > 16 && (Tk + 15) / 16 <= 20;
            if (s_rows == 32) {
                if (five) dscore_block<TV, 5, 2>(dC, V, P, key_len, dS, ds_rowsum, s_dp, b, i0, Tq, Tk, Dv, pitch);
                else dscore_block<TV, 4, 2>(dC, V, P, key_len, dS, ds_rowsum, s_dp, b, i0, Tq, Tk, Dv, pitch);
            } else {
                if (five) dscore_block<TV, 5, 1>(dC, V, P, key_len, dS, ds_rowsum, s_dp, b, i0, Tq, Tk, Dv, pitch);
                else dscore_block<TV, 4, 1>(dC, V, P, key_len, dS, ds_rowsum, s_dp, b, i0, Tq, Tk, Dv, pitch);
            }
        }
        return;
    }
    li -= spx * s_tiles;
    const int b = xcd + kXcd * (li / per_b), rem = li % per_b;
    if (b >= B) return;
    if constexpr (KT == 1) {
        dv_cols_block<KT>(P, dC, key_len, dV, Tq, Tk, Dv, b, rem, acc);
    } else if constexpr (KT == 2) {           // v_groups = column groups of 256, times the panels of 64 keys
        const int v_xt = (Dv + 255) / 256;
        dv_tile64(P, dC, key_len, dV, Tq, Tk, Dv, b, rem / v_xt, rem % v_xt, acc);
    } else {                                  // v_groups = column groups of 256, times the key tiles
        const int v_xt = (Dv + 255) / 256;
        pv_block<float, true>(P, dC, key_len, dV, Tq, Tk, Dv, b, rem / v_xt, rem % v_xt, acc);
    }
}

hipError_t launch_bwd_pre(const AttnShape &s, const float *dC, const void *V, const float *P, const int *key_len,
                          float *dS, float *ds_rowsum, int *order, float *dV, hipStream_t st, bool with_ds) {
    const int sorted = s.B <= kMaxSortedB ? 1 : 0;
    const int n_hs = (s.H + 63) / 64;
    const int fold = (sorted && (long long)s.B * n_hs <= 512) ? 1 : 0;   // recompute grid in one round
    // dS row tile: 32 rows on long key axes while three such blocks still fit a CU's LDS (the sample's V rows then
    // pass through half as many blocks), 16 otherwise
    const int s_rows = (s.Tk > kDsplitMaxTk && s.Tk <= kDs32MaxTk && s.Tq > 16) ? 32 : 16;
    const int s_tiles = with_ds ? (s.Tq + s_rows - 1) / s_rows : 0;
    // dV blocks per sample.  Short key axes (at most four key tiles, one per wave): a block owns 64 columns and all
    // keys, so its slice of dC is read once (dv_cols_block).  Up to 128 keys: a block per 16 keys and 256 columns
    // (pv_block); there the all-keys form was measured slower (3 to 12 % of this kernel at workloads 2 and 3: fewer,
    // longer blocks balance worse and a wave's batches of loads are too short to cover a trip to memory), and so
    // were panels of 64 keys (backward 139.5 -> 147 us at B = 128, T = 100: the second panel is half empty).
    // Beyond 128 keys, Tk a multiple of four: panels of 64 keys x 256 columns (dv_tile64; backward 635 -> 629 us
    // at B = 32, T = 300, H = 1024, where this launch now runs at 60 % of the matrix cores' fp32 peak).
    const int per_wave = ((s.Tk + 15) / 16 + 3) / 4;
    const int kt = per_wave <= 1 ? 1 : (s.Tk % 4 == 0 && s.Tk > kDsplitMaxTk ? 2 : 0);
    const int v_groups = kt == 1   ? (s.Dv + 63) / 64
                         : kt == 2 ? ((s.Dv + 255) / 256) * ((s.Tk + 63) / 64)
                                   : ((s.Dv + 255) / 256) * ((s.Tk + 15) / 16);
    const long long blocks = 1 + 8LL * ((s.B + 7) / 8) * (s_tiles + (long long)v_groups);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const int pitch16 = (s.Tk + 15) / 16 * 16 + 4;
    // short key axes: four planes of 16 rows, or (one round over d) the four waves' staging regions, which the
    // planes then share
    const size_t lds = s.Tk > kDsplitMaxTk ? (size_t)s_rows * pitch16 * sizeof(float)
                       : s.Dv <= 512       ? (size_t)4 * 16 * kStagePitch * sizeof(float)
                       : s.Dv <= 1024      ? (size_t)(4 * 16 * kStagePitch + 64 * pitch16) * sizeof(float)
                                           : (size_t)64 * pitch16 * sizeof(float);
#define ECHO_PRE_LAUNCH(TV, KT)                                                                                     \
    do {                                                                                                            \
        if (lds > 48 * 1024) { /* beyond the default dynamic LDS limit (up to 160 KB per block on gfx950) */        \
            static LdsGrants granted;                                                                               \
            hipError_t e = ensure_dynamic_lds((const void *)k_bwd_pre<TV, KT>, lds, granted);                       \
            if (e != hipSuccess) return e;                                                                          \
        }                                                                                                           \
        k_bwd_pre<TV, KT><<<(unsigned)blocks, 256, lds, st>>>(dC, (const TV *)V, P, key_len, dS, ds_rowsum, order, dV, \
                                                             s.B, sorted, fold, s.Tq, s.Tk, s.Dv, ds_pitch(s.Tk),  \
                                                             s_tiles, s_rows, v_groups, s.acc ? 1 : 0);                     \
    } while (0)
#define ECHO_PRE_KT(TV)                                 \
    switch (kt) {                                       \
        case 1: ECHO_PRE_LAUNCH(TV, 1); break;          \
        case 2: ECHO_PRE_LAUNCH(TV, 2); break;          \
        default: ECHO_PRE_LAUNCH(TV, 0); break;         \
    }
    if (s.bf16) {
        ECHO_PRE_KT(bf16_t)
    } else {
        ECHO_PRE_KT(float)
    }
#undef ECHO_PRE_KT
#undef ECHO_PRE_LAUNCH
    return hipGetLastError();
}

}  // namespace echo
