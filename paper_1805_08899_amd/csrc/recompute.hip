// B3: the fused recomputation kernel.  For every valid (b, i, j, h) it
// re-evaluates t = tanh(Qp[b,i,h] + Kp[b,j,h]) (Section 3.4: redo the cheap
// forward nodes when the backward pass starts; Section 6.1: the nodes on the
// recomputation path fused into one kernel) and accumulates
//     dQp[b,i,h] = v[h] sum_j dS[b,i,j] (1 - t^2)        (Section 3.2: tanh' = 1 - tanh^2)
//     dKp[b,j,h] = v[h] sum_i dS[b,i,j] (1 - t^2)
//     dv[h]     += sum_{i,j} dS[b,i,j] t                  (Eq. 2: needs the tanh map as the input of the v projection)
// without the B x Tq x Tk x H map ever existing in memory.
//
// A block owns one sample and one 64-wide slice of h; lanes run along h, so
// dS[b,i,j] is uniform over a wave and dQp, dKp, dv are plain per-lane sums.
// With r = 1 / (exp(2(q+k)) + 1):  t = 1 - 2r  and  1 - t^2 = 4 r (1 - r).
// Wave w owns query rows; all waves walk the keys together in tiles of RJ.
// The key tile (exponentials) and the dS tile are fetched one tile ahead and
// shared through LDS.  Per tile a wave adds its partial column sums into LDS, and after the
// barrier wave jj sums key jj of the tile over the waves in fixed order and
// owns that element of dKp for the whole kernel (first block of rows stores,
// later ones add), so no atomics are needed and results are reproducible.
//
// STASH reads t from a stored map instead (the keep-the-feature-map baseline,
// comparison only).
#include "common.hpp"
#include "kernels.hpp"

namespace echo {

constexpr int RC_RI = 8;      // query rows per wave and pass
constexpr int RC_RJ = 8;      // keys per tile (== kDsPad)
constexpr int RC_W = 8;       // waves per block (== RC_RJ: wave jj finishes key jj of a tile)
constexpr int RC_THREADS = 64 * RC_W;
static_assert(RC_RJ == kDsPad, "dS rows are padded to the key tile");
static_assert(RC_W == RC_RJ, "one finishing wave per key of a tile");
static_assert(RC_W == 8, "rows are dealt to eight waves");

enum RcMode { RC_FACTOR = 0, RC_EXACT = 1, RC_STASH = 2 };


// One RI x RJ register tile.  NI = number of live rows (compile time so the
// accumulators stay in registers and the NI*RJ chains interleave freely).
//   RC_FACTOR: fq = exp(2q), fk = exp(2k)        r = 1 / (fq fk + 1)
//   RC_EXACT : fq = 2 log2e q, fk = 2 log2e k    r = 1 / (exp2(fq + fk) + 1)
//   RC_STASH : t read from the stored map        r = (1 - t) / 2
// ds_tile points at dS[b, i0, j0] (wave-uniform values, zero at masked keys);
// t_tile at tmap[b, i0, 0, h] of this lane, kcol[c] = key index of column c
// clamped into the valid range.
template <int NI, int MODE, int NJ>
__device__ __forceinline__ void rc_tile(const float (&fq)[RC_RI], const float (&fk)[RC_RJ],
                                        const float *__restrict__ ds_tile, int pitch,
                                        const float *__restrict__ t_tile, size_t t_row, size_t t_key,
                                        const int (&kcol)[RC_RJ],
                                        float (&accQ)[RC_RI], float (&accK)[RC_RJ], float (&accV)[4]) {
    // Row by row; the eight evaluations of a row are issued as batches (multiply-adds, reciprocals, ...) so
    // that no instruction waits for the one before it.
#pragma unroll
    for (int a = 0; a < NI; ++a) {
        const float4 d0 = *reinterpret_cast<const float4 *>(ds_tile + a * pitch);
        const float4 d1 = NJ > 4 ? *reinterpret_cast<const float4 *>(ds_tile + a * pitch + 4) : d0;
        const float d[RC_RJ] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
        float r[NJ], u[NJ];
        if (MODE == RC_STASH) {
#pragma unroll
            for (int c = 0; c < NJ; ++c) r[c] = __builtin_fmaf(-0.5f, t_tile[a * t_row + kcol[c] * t_key], 0.5f);
        } else {
#pragma unroll
            for (int c = 0; c < NJ; ++c)
                r[c] = MODE == RC_FACTOR ? __builtin_fmaf(fq[a], fk[c], 1.0f) : fast_exp2(fq[a] + fk[c]) + 1.0f;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int c = 0; c < NJ; ++c) r[c] = fast_rcp(r[c]);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int c = 0; c < NJ; ++c) u[c] = __builtin_fmaf(-r[c], r[c], r[c]);      // r (1 - r) = (1 - t^2) / 4
        float q0 = 0.f, q1 = 0.f;
#pragma unroll
        for (int c = 0; c < NJ; c += 2) {
            accK[c] = __builtin_fmaf(d[c], u[c], accK[c]);
            q0 = __builtin_fmaf(d[c], u[c], q0);
            accV[c & 3] = __builtin_fmaf(d[c], r[c], accV[c & 3]);
            accK[c + 1] = __builtin_fmaf(d[c + 1], u[c + 1], accK[c + 1]);
            q1 = __builtin_fmaf(d[c + 1], u[c + 1], q1);
            accV[(c + 1) & 3] = __builtin_fmaf(d[c + 1], r[c + 1], accV[(c + 1) & 3]);
        }
        accQ[a] += q0 + q1;
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int MODE>
__device__ __forceinline__ void rc_tile_n(int ni, int live, const float (&fq)[RC_RI], const float (&fk)[RC_RJ],
                                          const float *__restrict__ ds_tile, int pitch,
                                          const float *__restrict__ t_tile, size_t t_row, size_t t_key,
                                          const int (&kcol)[RC_RJ],
                                          float (&accQ)[RC_RI], float (&accK)[RC_RJ], float (&accV)[4]) {
#define RC_CASE(N) \
    case N:                                                                                              \
        if (live <= 4) rc_tile<N, MODE, 4>(fq, fk, ds_tile, pitch, t_tile, t_row, t_key, kcol, accQ, accK, accV); \
        else rc_tile<N, MODE, RC_RJ>(fq, fk, ds_tile, pitch, t_tile, t_row, t_key, kcol, accQ, accK, accV);       \
        break;
    switch (ni) {
        RC_CASE(1) RC_CASE(2) RC_CASE(3) RC_CASE(4) RC_CASE(5) RC_CASE(6) RC_CASE(7) RC_CASE(8)
        default: break;
    }
#undef RC_CASE
}

// An element as loaded, and the number it stands for, as two steps: a load that sits in a guarded branch together
// with the first operation on its value (for bf16 the shift that widens it) makes the compiler wait for the load
// inside that branch, one trip to memory per load.  The raw form is what the load instruction delivers (bf16: the
// 16 bits, zero-extended); zero stands for zero in both.
template <typename T> struct RawElem;
template <> struct RawElem<float> {
    typedef float type;
    static __device__ __forceinline__ type load(const float *p, size_t i) { return p[i]; }
    static __device__ __forceinline__ float value(type r) { return r; }
};
template <> struct RawElem<bf16_t> {
    typedef unsigned type;
    static __device__ __forceinline__ type load(const bf16_t *p, size_t i) { return p[i].bits; }
    static __device__ __forceinline__ float value(type r) { return __uint_as_float(r << 16); }
};

template <typename T, bool STASH>
__global__ __launch_bounds__(RC_THREADS) void k_recompute(
    const T *__restrict__ Qp, const T *__restrict__ Kp, const T *__restrict__ v,
    const int *__restrict__ order, const float *__restrict__ dS, const float *__restrict__ ds_rowsum,
    const float *__restrict__ tmap, float *__restrict__ dQp, float *__restrict__ dKp, float *dv_part,
    unsigned long long *dv_flag, unsigned long long epoch, float *__restrict__ dv,
    int Tq, int Tk, int H, int pitch, int rows_per_pass, int acc) {
    // Key tile staged once per block, double buffered: exp(2k) for the factor
    // path, 2 log2e k for the exact path, and per key a flag "beyond the factor limit".
    __shared__ float s_fk[2][RC_RJ][64];
    __shared__ float s_sk[2][RC_RJ][64];
    __shared__ int s_kbig[2][RC_RJ];
    __shared__ __align__(16) float s_ds[2][RC_THREADS];     // dS of the pass rows x tile keys, [row][key]
    __shared__ float s_part[2][RC_W][RC_RJ][64];
    __shared__ float s_dv[RC_W][64];
    __shared__ float s_rowsum;
    __shared__ int s_seen[RC_W];

    // slot -> sample (the heaviest samples start first) and its clamped key length, packed by the ranking block
    const int packed = order[blockIdx.y];
    const int b = packed & 0xffff, L = packed >> 16;
    const int lane = lane_id(), w = wave_id();
    const int h = blockIdx.x * 64 + lane;
    const bool hv = h < H;
    const int hc = hv ? h : H - 1;
    // v of this lane's h: requested here, first touched behind the first loads of a pass (as a guarded load followed
    // by its scaling the compiler waited for it on the spot: a trip to memory before anything else had been requested)
    float v_raw = ld(v, hc);

    float *dQb = dQp ? dQp + (size_t)b * Tq * H : nullptr;
    float *dKb = dKp + (size_t)b * Tk * H;

    // masked keys: exact zeros (when adding to earlier decoder steps they hold zeros already)
    if (!acc)
        for (int j = L + w; j < Tk; j += RC_W)
            if (hv) dKb[(size_t)j * H + h] = 0.f;
    if (L == 0 && dQp) {                            // block-uniform
        for (int i = w; i < Tq; i += RC_W)
            if (hv) dQb[(size_t)i * H + h] = 0.f;
    }
    // sum of this sample's dS (zero in exact arithmetic): the part of sum dS t that comes from t = 1 - 2r.  The last
    // wave adds it up behind the first loads of the first pass, so that its rows are not a trip to memory late.
    auto sum_rows = [&]() {
        float rs = 0.f;
        for (int i = lane; i < Tq; i += 64) rs += ds_rowsum[(size_t)b * Tq + i];
        rs = wave_sum(rs);
        if (lane == 0) s_rowsum = rs;
    };
    if (L == 0 && w == RC_W - 1) sum_rows();

    float accV[4] = {0.f, 0.f, 0.f, 0.f};
    if (L > 0) {
        const T *qb = Qp + (size_t)b * Tq * H;
        const T *kb = Kp + (size_t)b * Tk * H;
        const float *dsb = dS + (size_t)b * Tq * pitch;
        const int n_jt = (L + RC_RJ - 1) / RC_RJ;

        // Tile staging, one tile ahead of the arithmetic.  Wave w fetches key w of the
        // tile (RC_W == RC_RJ) and thread t the dS element (row t / 8, key t % 8) of
        // the pass; the loads are issued before the current tile is evaluated and
        // committed to the other LDS buffer after it.
        const int t_row = threadIdx.x / RC_RJ, t_col = threadIdx.x % RC_RJ;
        typedef RawElem<T> Raw;
        typename Raw::type kx_raw = 0;
        float dx = 0.f;
        auto fetch = [&](int jt, int i_pass0, int nrows) {
            const int j = jt * RC_RJ + w;
            kx_raw = 0;
            if (!STASH && j < L) kx_raw = Raw::load(kb, (size_t)j * H + hc);
            dx = (t_row < nrows) ? dsb[(size_t)(i_pass0 + t_row) * pitch + jt * RC_RJ + t_col] : 0.f;
        };
        auto commit = [&](int jt, int buf) {
            const int j = jt * RC_RJ + w;
            s_ds[buf][threadIdx.x] = dx;
            if (STASH) return;
            asm volatile("" : "+v"(kx_raw));
            const float kx = Raw::value(kx_raw);
            s_sk[buf][w][lane] = kTwoLog2e * kx;
            s_fk[buf][w][lane] = (j < L) ? fast_exp2(kTwoLog2e * kx) : 0.f;
            const int big = __any(fabsf(kx) > kFactorLimit) ? 1 : 0;
            if (lane == 0) s_kbig[buf][w] = big;
        };

        int pass = 0;
        for (int i_pass0 = 0; i_pass0 < Tq; i_pass0 += rows_per_pass, ++pass) {
            const int nrows = min(rows_per_pass, Tq - i_pass0);
            const int r_lo = deal8_begin(nrows, w), r_hi = deal8_begin(nrows, w + 1);
            const int ni = r_hi - r_lo;              // 0..RC_RI
            const int i0 = i_pass0 + r_lo;

            fetch(0, i_pass0, nrows);
            float fq[RC_RI], sq[RC_RI], accQ[RC_RI];
            bool qbig = false;
            {
                typename Raw::type xr[RC_RI];
#pragma unroll
                for (int a = 0; a < RC_RI; ++a) {
                    xr[a] = 0;
                    if (!STASH && a < ni) xr[a] = Raw::load(qb, (size_t)(i0 + a) * H + hc);
                }
                if (pass == 0 && w == RC_W - 1) sum_rows();
                asm volatile("" : "+v"(v_raw));
                float x[RC_RI];
#pragma unroll
                for (int a = 0; a < RC_RI; ++a) {
                    asm volatile("" : "+v"(xr[a]));
                    x[a] = Raw::value(xr[a]);
                }
#pragma unroll
                for (int a = 0; a < RC_RI; ++a) {
                    accQ[a] = 0.f;
                    qbig |= fabsf(x[a]) > kFactorLimit;
                    sq[a] = kTwoLog2e * x[a];
                    fq[a] = fast_exp2(sq[a]);
                }
            }
            const float v4 = hv ? 4.f * v_raw : 0.f;
            const bool wave_qbig = __any(qbig);
            commit(0, 0);
            lds_barrier();

            for (int jt = 0; jt < n_jt; ++jt) {
                const int buf = jt & 1;
                const int j0 = jt * RC_RJ;
                const bool more = jt + 1 < n_jt;
                // valid keys of this tile: a last tile with at most four evaluates half the columns (finer steps
                // make the backward pass alone faster, but the code grows and forward + backward, which alternate
                // in a training step, get slower)
                const int live = L - j0;
                if (more) fetch(jt + 1, i_pass0, nrows);
                float accK[RC_RJ], fk[RC_RJ];
                int kcol[RC_RJ];
#pragma unroll
                for (int c = 0; c < RC_RJ; ++c) {
                    accK[c] = 0.f;
                    kcol[c] = min(j0 + c, L - 1);
                }
                const float *ds_tile = &s_ds[buf][r_lo * RC_RJ];     // wave-uniform reads, pitch RC_RJ
                if (STASH) {
                    const float *t_tile = tmap + (((size_t)b * Tq + i0) * Tk) * H + hc;
#pragma unroll
                    for (int c = 0; c < RC_RJ; ++c) fk[c] = 0.f;
                    rc_tile_n<RC_STASH>(ni, live, fq, fk, ds_tile, RC_RJ, t_tile, (size_t)Tk * H, (size_t)H, kcol, accQ, accK,
                                        accV);
                } else {
                    int kbig = 0;
#pragma unroll
                    for (int c = 0; c < RC_RJ; ++c) kbig |= s_kbig[buf][c];
                    if (!(wave_qbig || kbig)) {
#pragma unroll
                        for (int c = 0; c < RC_RJ; ++c) fk[c] = s_fk[buf][c][lane];
                        rc_tile_n<RC_FACTOR>(ni, live, fq, fk, ds_tile, RC_RJ, nullptr, 0, 0, kcol, accQ, accK, accV);
                    } else {
#pragma unroll
                        for (int c = 0; c < RC_RJ; ++c) fk[c] = s_sk[buf][c][lane];
                        rc_tile_n<RC_EXACT>(ni, live, sq, fk, ds_tile, RC_RJ, nullptr, 0, 0, kcol, accQ, accK, accV);
                    }
                }
                if (more) commit(jt + 1, buf ^ 1);
#pragma unroll
                for (int c = 0; c < RC_RJ; ++c) s_part[buf][w][c][lane] = accK[c];
                lds_barrier();
                // wave w finishes key j0 + w of this tile: sum over the waves in fixed order
                const int j = j0 + w;
                float tot = 0.f;
#pragma unroll
                for (int w2 = 0; w2 < RC_W; ++w2) tot += s_part[buf][w2][w][lane];
                if (j < L && hv) {
                    float *dst = dKb + (size_t)j * H + h;
                    const float val = v4 * tot;
                    if (pass == 0 && !acc) store_streaming(dst, val);
                    else *dst = *dst + val;
                }
            }
            if (hv && dQp) {
#pragma unroll
                for (int a = 0; a < RC_RI; ++a)
                    if (a < ni) store_streaming(&dQb[(size_t)(i0 + a) * H + h], v4 * accQ[a]);
            }
            lds_barrier();   // the next pass restages buffer 0 and reuses s_part
        }
    }

    // dv partial of this sample: sum dS t = sum dS - 2 sum dS r
    s_dv[w][lane] = (accV[0] + accV[1]) + (accV[2] + accV[3]);
    lds_barrier();
    const int n_slots = gridDim.y;
    unsigned long long *flags = dv_flag + (size_t)blockIdx.x * n_slots;      // of this slice of h, one per slot
    if (w == 0) {
        if (hv) {
            float tot = 0.f;
#pragma unroll
            for (int w2 = 0; w2 < RC_W; ++w2) tot += s_dv[w2][lane];
            store_agent(&dv_part[(size_t)b * H + h], __builtin_fmaf(-2.f, tot, s_rowsum));
        }
        // B4 without a launch of its own: the part is published (written through, awaited, then flagged with
        // this launch's number), and the block of the last slot, which starts last and holds the lightest
        // sample, adds the parts of its slice of h once all of them are flagged.
        wait_all_memory_ops();
        if (lane == 0) store_agent(&flags[blockIdx.y], epoch);
    }
    if ((int)blockIdx.y != n_slots - 1) return;
    lds_barrier();                                   // s_dv is reused below
    const long long t_wait0 = wall_clock64();
    int seen = 1;
    for (int s0 = threadIdx.x; s0 < n_slots; s0 += RC_THREADS) {
        while (load_agent(&flags[s0]) != epoch) {
            __builtin_amdgcn_s_sleep(4);
            if (wall_clock64() - t_wait0 > kSpinLimitTicks) {
                seen = 0;
                break;
            }
        }
    }
    // samples in index order, eight groups of them added group by group: the order of additions is fixed
    float part = 0.f;
    s_seen[w] = __all(seen) ? 1 : 0;
    lds_barrier();
    bool all_seen = true;
#pragma unroll
    for (int w2 = 0; w2 < RC_W; ++w2) all_seen = all_seen && s_seen[w2] != 0;
    if (hv && all_seen) {
        for (int b0 = w; b0 < n_slots; b0 += 8 * RC_W) {
            float x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                x[u] = (b0 + RC_W * u < n_slots) ? load_agent(&dv_part[(size_t)(b0 + RC_W * u) * H + h]) : 0.f;
#pragma unroll
            for (int u = 0; u < 8; ++u) part += x[u];
        }
    }
    s_dv[w][lane] = part;
    lds_barrier();
    if (w == 0 && hv) {
        float tot = 0.f;
#pragma unroll
        for (int w2 = 0; w2 < RC_W; ++w2) tot += s_dv[w2][lane];
        if (!all_seen) tot = __builtin_nanf("");      // a part never arrived: make the failure visible
        dv[h] = acc ? dv[h] + tot : tot;
    }
    // leave the flags cleared: a replay of a captured launch carries the same launch number
    for (int s0 = threadIdx.x; s0 < n_slots; s0 += RC_THREADS) store_agent(&flags[s0], 0ull);
}


template <typename T>
static hipError_t launch_recompute_t(const AttnShape &s, const void *Qp, const void *Kp, const void *v,
                                     const int *order, const float *dS, const float *ds_rowsum, const float *tmap,
                                     float *dQp, float *dKp, float *dv_part, unsigned long long *dv_flag,
                                     unsigned long long epoch, float *dv, hipStream_t st) {
    const int max_rows = RC_W * RC_RI;
    const int n_pass = (s.Tq + max_rows - 1) / max_rows;
    // full passes of 64 rows first, the remainder last: with the rows split evenly over the passes, waves of 7 and of 8
    // rows meet at every tile's barrier (100 rows: 64 + 36 instead of 50 + 50; backward 141.5 -> 139.8 us at B = 128)
    const int rows_per_pass = s.Tq > max_rows ? max_rows : s.Tq;
    (void)n_pass;
    dim3 grid((s.H + 63) / 64, s.B);
    if (tmap)
        k_recompute<T, true><<<grid, RC_THREADS, 0, st>>>((const T *)Qp, (const T *)Kp, (const T *)v, order, dS,
                                                          ds_rowsum, tmap, dQp, dKp, dv_part, dv_flag, epoch, dv,
                                                          s.Tq, s.Tk, s.H, ds_pitch(s.Tk), rows_per_pass,
                                                          s.acc ? 1 : 0);
    else
        k_recompute<T, false><<<grid, RC_THREADS, 0, st>>>((const T *)Qp, (const T *)Kp, (const T *)v, order, dS,
                                                           ds_rowsum, tmap, dQp, dKp, dv_part, dv_flag, epoch, dv,
                                                           s.Tq, s.Tk, s.H, ds_pitch(s.Tk), rows_per_pass,
                                                           s.acc ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_recompute(const AttnShape &s, const void *Qp, const void *Kp, const void *v, const int *order,
                            const float *dS, const float *ds_rowsum, const float *tmap, float *dQp, float *dKp,
                            float *dv_part, unsigned long long *dv_flag, unsigned long long epoch, float *dv,
                            hipStream_t st) {
    return s.bf16 ? launch_recompute_t<bf16_t>(s, Qp, Kp, v, order, dS, ds_rowsum, tmap, dQp, dKp, dv_part, dv_flag,
                                               epoch, dv, st)
                  : launch_recompute_t<float>(s, Qp, Kp, v, order, dS, ds_rowsum, tmap, dQp, dKp, dv_part, dv_flag,
                                              epoch, dv, st);
}

}  // namespace echo
