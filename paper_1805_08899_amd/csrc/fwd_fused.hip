// Forward pass in one kernel: scores, masked softmax and context for a tile of
// query rows of one sample, without S ever reaching memory
// (Section 2, attention steps 1-2; Section 4.1 scoring function; Section 6.1:
// one fused kernel instead of many small ones, fewer launches and accesses).
//
// Block = (sample b, up to RT = 8 NG query rows), W waves: eight, or four in streaming mode at H <= 512 (four
// such blocks share a CU and are in different phases of their lives, which keeps the vector units fed).
//   A  exp(2q) / v of the rows and 1 / v go to LDS (taken once per block).
//   B  the valid keys are dealt to the waves in W contiguous shares that differ by at most one key;
//      a wave walks its share in passes of up to four keys.  A lane owns four
//      consecutive h of every 256-wide slice, so a key row arrives as one
//      16-byte load per lane (every K element is exponentiated once per block)
//      and a staged query row as one 16-byte LDS read.
//      With r = 1 / (exp(2(q+k)) + 1), tanh = 1 - 2r, the score is sum_h v - 2 sum_h v r, and the first
//      term drops out of the softmax.  v r = 1 / a with a = 1/v + (exp(2q)/v) exp(2k): one multiply-add.
//      Two neighbouring h share one reciprocal: 1/a0 + 1/a1 = (a0 + a1) / (a0 a1), so per row, key and
//      pair of h the loop issues 2 fma, 1 add, 1 mul, 1 rcp, 1 fma.
//      A pass finishes with one transposing wave reduction of its rows x keys tile.  A pass whose
//      operands could leave the range in which a0 a1 stays finite is redone by a small exact routine
//      that exponentiates the sum.
//   C  the waves normalise the rows (softmax over the valid keys) and write P.
//   D  context = P V on the matrix cores: v_mfma_f32_4x4x1 treats the 64 lanes
//      as 16 column groups of 4, so a lane owns one output column and reads V
//      rows with plain coalesced loads (in batches of rows, one batch ahead; all rows at once,
//      before the softmax, when the key axis is short: ContextAllRows; two waves per group of 256
//      columns with half of the keys each when there are twice as many waves as groups: ContextSplitKeys).
//
// A block's whole pass is short compared with a trip to memory, so loads are
// issued well before they are consumed: the first key slice leaves before the
// query rows are staged, key slices run one ahead of the arithmetic across
// pass boundaries, and the first value rows leave before the softmax.
//
// Placement.  The hardware hands blocks to the XCDs round-robin.  For small
// batches one wave of the block ranks the samples by valid keys (lengths in
// registers) and hands the block's sample to the other waves through LDS; samples go to the XCDs in snake order (equal
// work per XCD, all tiles of a sample share one L2) and, when two blocks share
// a CU, gives the CUs that hold one block the heaviest tiles and pairs heavy
// with light tiles on the others; with more rounds of blocks the heaviest
// simply start first.  The mapping only moves work around; results do not
// depend on it.
#include <type_traits>

#include "common.hpp"
#include "kernels.hpp"

namespace echo {

typedef float f32x4 __attribute__((ext_vector_type(4)));


constexpr int FW_W = 8;          // waves per block in row mode (deal8_begin deals the keys to eight)
constexpr int FW_W_STREAM = 4;   // waves per block in streaming mode when H <= 512: four blocks per CU instead of
                                 // two, so that more blocks are in different phases at any time (placement, staging,
                                 // softmax and context wait on memory; only the score loop fills the vector units)
constexpr int FW_NJ = 4;         // keys per wave and pass (register tile columns)
constexpr int FW_SS = 256;       // h per slice: four per lane
constexpr int FW_XCD = 8;        // blockIdx.x mod 8 selects the XCD
constexpr int FW_CU_PER_XCD = 32;
constexpr int FW_KB = 16;        // value rows per batch in the context phase (two batches in flight per wave)
constexpr int FW_MAX_RANKED_B = 128;   // the in-kernel ranking keeps two lengths per lane
constexpr int FW_ROW_REGS = 16;  // row mode: 16-byte registers a wave spends on its keys (keys x slices)

// row mode: the longest key share a wave can hold with ns slices of h (1 stands in for streaming mode, ns = 0)
constexpr int fw_row_max_keys(int ns) { return ns <= 0 ? 1 : (FW_ROW_REGS / ns > 8 ? 8 : FW_ROW_REGS / ns); }

__device__ __forceinline__ float comp(const float4 &x, int c) { return c == 0 ? x.x : c == 1 ? x.y : c == 2 ? x.z : x.w; }

// Four consecutive elements of a key row exactly as they were loaded: one 16- or 8-byte register group that stays
// whole from the load to pin().  Row mode loads its keys under uniform branches (a wave requests only its own
// keys); if the loaded value were taken apart or converted right away, the compiler would merge those pieces with
// the other branch's zeros inside the branch and wait for every key in turn behind its load: one trip to memory per
// key instead of one for all.  pin() marks the place from where the value may be used.
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
template <typename T> struct RawKey;
template <> struct RawKey<float> {
    f32x4 v;
    __device__ __forceinline__ void load(const float *p, size_t i) { v = *reinterpret_cast<const f32x4 *>(p + i); }
    __device__ __forceinline__ void zero() { v = f32x4{0.f, 0.f, 0.f, 0.f}; }
    __device__ __forceinline__ void pin() { asm("" : "+v"(v)); }
    __device__ __forceinline__ float4 get() const { return make_float4(v.x, v.y, v.z, v.w); }
};
template <> struct RawKey<bf16_t> {
    u32x2 v;
    __device__ __forceinline__ void load(const bf16_t *p, size_t i) { v = *reinterpret_cast<const u32x2 *>(p + i); }
    __device__ __forceinline__ void zero() { v = u32x2{0u, 0u}; }
    __device__ __forceinline__ void pin() { asm("" : "+v"(v)); }
    __device__ __forceinline__ float4 get() const {
        return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u),
                           __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u));
    }
};

// Pairs of reciprocals share one division (see B at the top): the product a0 a1 must stay finite.
// |a| <= max|1/v| + max|exp(2q)/v| max exp(2k); a pass is evaluated by the factor path only while this
// bound is below kPairLimit = sqrt(FLT_MAX) (with a little room).  An entry of v below kTinyV in magnitude
// is taken as zero (it changes a score by less than 1e-18): its 1/v is replaced by kHugeC and its
// exp(2q)/v by 0, so that the pair still evaluates to the other entry's term.
constexpr float kPairLimit = 1.8e19f;
constexpr float kTinyV = 1e-18f;
constexpr float kHugeC = 1e18f;

// One row of the tile against NJ keys for the four h of a lane: t = 1/v + (exp(2q)/v) exp(2k), then per pair
// of h one sum, one product, one reciprocal and one multiply-add into acc.  The evaluations are issued in
// batches so that no instruction waits for the one before it.  fk[q][c]: exp(2k) of key c at the lane's q-th h.
template <int NJ>
__device__ __forceinline__ void fw_row_keys(const float4 &fq, const float4 &cv, const float (&fk)[4][NJ], float (&acc)[NJ]) {
    float t[4][NJ], sm[2][NJ], pr[2][NJ];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int c = 0; c < NJ; ++c) t[q][c] = __builtin_fmaf(comp(fq, q), fk[q][c], comp(cv, q));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
        for (int c = 0; c < NJ; ++c) {
            sm[h2][c] = t[2 * h2][c] + t[2 * h2 + 1][c];
            pr[h2][c] = t[2 * h2][c] * t[2 * h2 + 1][c];
        }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
        for (int c = 0; c < NJ; ++c) pr[h2][c] = fast_rcp(pr[h2][c]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
        for (int c = 0; c < NJ; ++c) acc[c] = __builtin_fmaf(sm[h2][c], pr[h2][c], acc[c]);
    __builtin_amdgcn_sched_barrier(0);
}

// The keys of one wave as a stream of slices: pass p covers keys j0(p) .. j0(p+1), slice s the columns
// 256 s + 4 lane .. + 3.  `cur` is the slice about to be consumed; once its values have been used advance()
// issues the loads of the following slice into the same registers, a whole slice of arithmetic ahead of their
// use.  Rows past a pass's last key repeat it.
template <typename T>
struct KeyStream {
    const T *kb;
    int H, lane4, k_lo, npass, NS;
    int base, extra;                    // pass p has base + (p < extra) keys
    int p_f, s_f;                       // slice that the next fetch will load
    float4 cur[FW_NJ];

    __device__ __forceinline__ void init(const T *kb_, int H_, int lane, int k_lo_, int nk, int NS_) {
        kb = kb_;
        H = H_;
        lane4 = 4 * lane;
        k_lo = nk > 0 ? k_lo_ : 0;        // a wave without keys loads key 0 (its own first key may be row L)
        NS = NS_;
        npass = (nk + FW_NJ - 1) / FW_NJ;
        const int np = max(npass, 1);
        // the same in all lanes, but the division runs on the vector unit: back to scalar registers, so that
        // everything derived from it (pass bounds, row addresses) is scalar arithmetic
        base = __builtin_amdgcn_readfirstlane(nk / np);
        extra = nk - base * np;
        p_f = 0;
        s_f = 0;
    }
    __device__ __forceinline__ int pass_begin(int p) const { return k_lo + p * base + min(p, extra); }

    // No branches here: past the last slice the loads simply repeat it (a wave without keys reads key 0,
    // which exists because the block has at least one valid key), so the loads in flight never meet a
    // control-flow join and stay in flight while the previous slice is being evaluated.
    __device__ __forceinline__ void fetch() {
        // the stream position is the same in all lanes; taken through scalar registers so that the pass bounds
        // and row addresses below are scalar arithmetic (the compiler otherwise carries them per lane)
        p_f = __builtin_amdgcn_readfirstlane(p_f);
        s_f = __builtin_amdgcn_readfirstlane(s_f);
        const int pc = min(p_f, max(npass, 1) - 1);
        const int j0 = pass_begin(pc), j1 = max(pass_begin(pc + 1), j0 + 1);
        // columns past H: the load repeats the row's last four values; exp(2q)/v is 0 and 1/v is kHugeC
        // there, so they add nothing
        const unsigned hc = (unsigned)min(s_f * FW_SS + lane4, H - 4);
#pragma unroll
        for (int c = 0; c < FW_NJ; ++c) {
            // row address from scalars, column from the lane: the load takes them as base and offset
            const T *row = kb + (size_t)(unsigned)(min(j0 + c, j1 - 1) * H);
            cur[c] = ld4(row, (size_t)hc);
        }
        const bool wrap = s_f + 1 == NS;
        s_f = wrap ? 0 : s_f + 1;
        p_f = wrap ? min(p_f + 1, npass) : p_f;
    }
    __device__ __forceinline__ void start() { fetch(); }
    __device__ __forceinline__ void advance() { fetch(); }
};

// Streaming mode, one pass of one wave: NJ keys starting at column jcol0 of the score tile, all rows of the
// block, all slices of h, factor path only.  s_e: LDS rows of exp(2q)/v, pitch Hp; s_c: 1/v.  NI > 0: exactly
// NI rows are live, known at compile time (no per-row branches, the next row's LDS read is issued a row ahead);
// NI == 0: the first ni.  What is written is the score without its key-independent term: -2 sum_h v r.
// qe_max, c_max: the block's largest |exp(2q)/v| and |1/v|.  Returns true if the operands may leave the
// range of the factor path, in which case nothing was written and the caller must redo the pass exactly.
template <typename T, int NG, int NJ, int NI>
__device__ __forceinline__ bool fw_pass(const float *__restrict__ s_e, const float *__restrict__ s_c, int Hp, int ni,
                                        KeyStream<T> &ks, float qe_max, float c_max, float *__restrict__ s_S,
                                        int spitch, int jcol0) {
    constexpr int RT = 8 * NG;
    constexpr bool FULL = NI > 0;
    constexpr int NR = FULL ? NI : RT;       // rows the unrolled loops visit
    const int lane = lane_id();
    float acc[RT][NJ];
#pragma unroll
    for (int a = 0; a < RT; ++a)
#pragma unroll
        for (int c = 0; c < NJ; ++c) acc[a][c] = 0.f;
    float kmax = 0.f;                        // largest exp(2k) this lane met

    for (int s = 0; s < ks.NS; ++s) {
        float fk[4][NJ];
#pragma unroll
        for (int c = 0; c < NJ; ++c) {
#pragma unroll
            for (int q = 0; q < 4; ++q) fk[q][c] = fast_exp2(kTwoLog2e * comp(ks.cur[c], q));
            kmax = fmaxf(fmaxf(kmax, fk[0][c]), fmaxf(fk[1][c], fmaxf(fk[2][c], fk[3][c])));
        }
        ks.advance();
        const float4 cv = *reinterpret_cast<const float4 *>(s_c + s * FW_SS + 4 * lane);
        const float *e_col = s_e + s * FW_SS + 4 * lane;
        float4 fq_next = *reinterpret_cast<const float4 *>(e_col);
#pragma unroll
        for (int a = 0; a < NR; ++a) {
            if (FULL || a < ni) {
                float4 fq;
                if (FULL) {
                    fq = fq_next;
                    if (a + 1 < NR) fq_next = *reinterpret_cast<const float4 *>(e_col + (a + 1) * Hp);
                } else {
                    fq = *reinterpret_cast<const float4 *>(e_col + a * Hp);
                }
                fw_row_keys<NJ>(fq, cv, fk, acc[a]);
            }
        }
    }
    // the negation also sends a NaN bound (NaN or infinite operands) to the exact path
    if (__any(!(__builtin_fmaf(qe_max, kmax, c_max) < kPairLimit))) return true;
    // per lane first, then one transposing reduction for the whole tile
    constexpr int NP = RT * NJ;
    constexpr int NPOW = NP <= 8 ? 8 : NP <= 16 ? 16 : NP <= 32 ? 32 : 64;
    float flat[NPOW];
#pragma unroll
    for (int p = 0; p < NPOW; ++p) {
        const int a = p / NJ, c = p % NJ;
        flat[p] = p < NP ? acc[a < RT ? a : 0][c] : 0.f;
    }
    const float tot = wave_transpose_sum<NPOW>(flat);
    const int p = lane / (64 / NPOW);
    if ((lane % (64 / NPOW)) == 0 && p < NP) {
        const int a = p / NJ, c = p % NJ;
        if (a < ni) s_S[a * spitch + jcol0 + c] = -2.f * tot;
    }
    return false;
}

// The same tile with r taken from the exponential of the sum: correct for any finite input.
// Straightforward loops; only reached for operands beyond the range of the factor path.
template <typename T>
__device__ __noinline__ void fw_pass_exact(const T *__restrict__ qrow0, int ni, const T *__restrict__ krow0, int nj,
                                           int H, const T *__restrict__ v, float *__restrict__ s_S, int spitch,
                                           int jcol0) {
    const int lane = lane_id();
    for (int a = 0; a < ni; ++a) {
        for (int c = 0; c < nj; ++c) {
            float acc = 0.f;
            for (int h = lane; h < H; h += 64) {
                const float sq = kTwoLog2e * ld(qrow0, (size_t)a * H + h);
                const float sk = kTwoLog2e * ld(krow0, (size_t)c * H + h);
                acc = __builtin_fmaf(ld(v, h), r_from_sum(sq, sk), acc);
            }
            acc = wave_sum(acc);
            if (lane == 0) s_S[a * spitch + jcol0 + c] = -2.f * acc;
        }
    }
}

// Row mode, for key shares small enough to sit in registers: NK keys x NS slices of exp(2k) per lane, loaded
// once (raw: the values as loaded before the staging barrier; this call takes keys C0 .. C0 + NK - 1 of them); then
// a plain loop over the tile's rows, each row against all NK keys, ending in one transposing reduction of the row's NK sums.  The loop body is short
// and runs ni times, where streaming mode spends most of a short block's life in code it runs once.
// Returns true (nothing written) if the operands may leave the range of the factor path.
template <typename T, int NS, int NKM, int NK, int C0 = 0>
__device__ __forceinline__ bool fw_rows(const RawKey<T> (&raw)[NS][NKM], const float *__restrict__ s_e,
                                        const float *__restrict__ s_c, int Hp, int ni, float qe_max, float c_max,
                                        float *__restrict__ s_S, int spitch, int jcol0) {
    const int lane = lane_id();
    float fk[NS][4][NK];
    float kmax = 0.f;
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int c = 0; c < NK; ++c) {
            const float4 kx = raw[s][C0 + c].get();
#pragma unroll
            for (int q = 0; q < 4; ++q) fk[s][q][c] = fast_exp2(kTwoLog2e * comp(kx, q));
            kmax = fmaxf(fmaxf(kmax, fk[s][0][c]), fmaxf(fk[s][1][c], fmaxf(fk[s][2][c], fk[s][3][c])));
        }
    if (__any(!(__builtin_fmaf(qe_max, kmax, c_max) < kPairLimit))) return true;
    constexpr int NPOW = NK <= 1 ? 1 : NK <= 2 ? 2 : NK <= 4 ? 4 : 8;
    const float *e_col = s_e + 4 * lane;
    const float *c_col = s_c + 4 * lane;
    float4 fq = *reinterpret_cast<const float4 *>(e_col);
    float4 cv = *reinterpret_cast<const float4 *>(c_col);
    for (int a = 0; a < ni; ++a) {
        float acc[NK];
#pragma unroll
        for (int c = 0; c < NK; ++c) acc[c] = 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            // operands of the next slice (of the next row after the last slice; the row past the last one
            // repeats it) are requested before this slice is evaluated
            const int a2 = s + 1 < NS ? a : min(a + 1, ni - 1), s2 = s + 1 < NS ? s + 1 : 0;
            const float4 fq2 = *reinterpret_cast<const float4 *>(e_col + a2 * Hp + s2 * FW_SS);
            const float4 cv2 = *reinterpret_cast<const float4 *>(c_col + s2 * FW_SS);
            if constexpr (NK <= 4) {
                fw_row_keys<NK>(fq, cv, fk[s], acc);
            } else {                         // groups of two keys so that the temporaries stay few
#pragma unroll
                for (int c0 = 0; c0 < NK; c0 += 2) {
                    if (c0 + 1 < NK) {
                        float f2[4][2], a2[2] = {acc[c0], acc[c0 + 1]};
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            f2[q][0] = fk[s][q][c0];
                            f2[q][1] = fk[s][q][c0 + 1];
                        }
                        fw_row_keys<2>(fq, cv, f2, a2);
                        acc[c0] = a2[0];
                        acc[c0 + 1] = a2[1];
                    } else {
                        float f1[4][1], a1[1] = {acc[c0]};
#pragma unroll
                        for (int q = 0; q < 4; ++q) f1[q][0] = fk[s][q][c0];
                        fw_row_keys<1>(fq, cv, f1, a1);
                        acc[c0] = a1[0];
                    }
                }
            }
            fq = fq2;
            cv = cv2;
        }
        {
            float flat[NPOW];
#pragma unroll
            for (int c = 0; c < NPOW; ++c) flat[c] = c < NK ? acc[c < NK ? c : 0] : 0.f;
            const float tot = wave_transpose_sum<NPOW>(flat);
            const int c = lane / (64 / NPOW);
            if ((lane % (64 / NPOW)) == 0 && c < NK) s_S[a * spitch + jcol0 + c] = -2.f * tot;
        }
    }
    return false;
}

template <typename T, int NS, int NKM>
__device__ __forceinline__ bool fw_rows_n(int nk, const RawKey<T> (&raw)[NS][NKM], const float *__restrict__ s_e,
                                          const float *__restrict__ s_c, int Hp, int ni, float qe_max, float c_max,
                                          float *__restrict__ s_S, int spitch, int jcol0) {
    // More than twelve 16-byte groups of exponentials (keys x slices) do not fit the registers next to the row
    // loop's operands: the loop would fetch them back from scratch memory row after row.  Such a share is
    // evaluated as two halves, each with its own loop over the rows.
#define FW_ROWS_CASE(N)                                                                                       \
    case N:                                                                                                   \
        if constexpr (N <= NKM && NS * N <= 12) {                                                             \
            return fw_rows<T, NS, NKM, N>(raw, s_e, s_c, Hp, ni, qe_max, c_max, s_S, spitch, jcol0);          \
        } else if constexpr (N <= NKM) {                                                                      \
            constexpr int A = (N + 1) / 2;                                                                    \
            const bool r1 = fw_rows<T, NS, NKM, A, 0>(raw, s_e, s_c, Hp, ni, qe_max, c_max, s_S, spitch, jcol0);         \
            const bool r2 = fw_rows<T, NS, NKM, N - A, A>(raw, s_e, s_c, Hp, ni, qe_max, c_max, s_S, spitch, jcol0 + A); \
            return r1 || r2;                                                                                  \
        }                                                                                                     \
        break;
    switch (nk) {
        FW_ROWS_CASE(1) FW_ROWS_CASE(2) FW_ROWS_CASE(3) FW_ROWS_CASE(4)
        FW_ROWS_CASE(5) FW_ROWS_CASE(6) FW_ROWS_CASE(7) FW_ROWS_CASE(8)
        default: break;
    }
#undef FW_ROWS_CASE
    return false;                            // nk == 0: nothing to do
}

// Context rows = P V on the matrix cores.  One 4x4x1 MFMA multiplies 4 rows of P (replicated over the 16 lane
// groups) with one V value per lane, so a lane owns an output column; with CPL > 1 a lane owns CPL neighbouring
// columns, loaded in one 8- or 16-byte piece and fed to CPL products, and a wave takes 64 CPL columns at a time.
// The batches of value rows of all of a wave's column groups form one sequence; the loads of the next batch are
// issued before the current one is multiplied.  Keys past L carry P = 0, the last valid row stands in for them;
// no branches around the loads, so that they stay in flight across the arithmetic of the batch before.
// Rows of a matrix read through a buffer descriptor: element address = base + vector byte offset + scalar byte offset,
// both 32-bit, range-checked by the hardware against the n_elems elements the descriptor covers (a load past them
// returns zero).  The descriptor's last word is the raw 32-bit data format of this architecture family.
template <typename T> struct BufferRows {
    __amdgpu_buffer_rsrc_t rsrc;
    __device__ __forceinline__ BufferRows(const T *base, unsigned n_elems)
        : rsrc(__builtin_amdgcn_make_buffer_rsrc(const_cast<T *>(base), 0, (int)(n_elems * (unsigned)sizeof(T)),
                                                  0x00020000)) {}
    // the element as loaded (16-bit types: the bits, zero-extended); value() turns it into the number.  Two steps so
    // that nothing but the load sits where the loads are issued (an operation on the loaded value there makes the
    // compiler wait for every load in turn)
    using Raw = std::conditional_t<sizeof(T) == 4, float, unsigned short>;
    __device__ __forceinline__ Raw load_raw(unsigned v_off, unsigned s_off) const {
        if constexpr (sizeof(T) == 4) {
            return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, v_off, s_off, 0));
        } else {
            return __builtin_amdgcn_raw_buffer_load_b16(rsrc, v_off, s_off, 0);
        }
    }
    // (16-bit types: the empty statement keeps the conversion behind whatever barrier precedes the call)
    static __device__ __forceinline__ float value(Raw raw) {
        if constexpr (sizeof(T) == 4) {
            return raw;
        } else {
            asm volatile("" : "+v"(raw));
            return __uint_as_float((unsigned)raw << 16);
        }
    }
};

// CPL consecutive columns of one row as they come from memory through a buffer descriptor (f32: CPL words;
// 16-bit types: CPL / 2 words, one for CPL = 1).  Loading and converting are separate steps: see BufferRows.
template <typename T, int CPL> struct RowPiece {
    static constexpr int kBytes = CPL * (int)sizeof(T);
    static constexpr int NW = (kBytes + 3) / 4;
    unsigned w[NW];
    __device__ __forceinline__ void load(const BufferRows<T> &rows, unsigned v_off, unsigned s_off) {
        if constexpr (kBytes == 2) {
            w[0] = __builtin_amdgcn_raw_buffer_load_b16(rows.rsrc, v_off, s_off, 0);
        } else if constexpr (kBytes == 4) {
            w[0] = __builtin_amdgcn_raw_buffer_load_b32(rows.rsrc, v_off, s_off, 0);
        } else if constexpr (kBytes == 8) {
            const auto x = __builtin_amdgcn_raw_buffer_load_b64(rows.rsrc, v_off, s_off, 0);
            w[0] = x[0];
            w[1] = x[1];
        } else {
            static_assert(kBytes == 16, "one to four columns of 2 or 4 bytes");
            const auto x = __builtin_amdgcn_raw_buffer_load_b128(rows.rsrc, v_off, s_off, 0);
            w[0] = x[0];
            w[1] = x[1];
            w[2] = x[2];
            w[3] = x[3];
        }
    }
    // 16-bit types: call before value(), at the place where the conversions may begin
    __device__ __forceinline__ void pin() {
        if constexpr (sizeof(T) == 2) {
#pragma unroll
            for (int i = 0; i < NW; ++i) asm volatile("" : "+v"(w[i]));
        }
    }
    __device__ __forceinline__ float value(int c) const {
        if constexpr (sizeof(T) == 4) return __uint_as_float(w[c]);
        else if constexpr (CPL == 1) return __uint_as_float(w[0] << 16);
        else return __uint_as_float((c & 1) ? (w[c >> 1] & 0xffff0000u) : (w[c >> 1] << 16));
    }
};

template <int CPL> struct ColVec;
template <> struct ColVec<1> {
    static __device__ __forceinline__ void load(const float *p, size_t i, float (&d)[1]) { d[0] = p[i]; }
    static __device__ __forceinline__ void load(const bf16_t *p, size_t i, float (&d)[1]) { d[0] = ld(p, i); }
    static __device__ __forceinline__ void store(float *p, const float (&x)[1]) { store_streaming(p, x[0]); }
};
template <> struct ColVec<2> {
    static __device__ __forceinline__ void load(const float *p, size_t i, float (&d)[2]) {
        const float2 x = *reinterpret_cast<const float2 *>(p + i);
        d[0] = x.x;
        d[1] = x.y;
    }
    static __device__ __forceinline__ void load(const bf16_t *p, size_t i, float (&d)[2]) {
        const uint32_t u = *reinterpret_cast<const uint32_t *>(p + i);
        d[0] = __uint_as_float(u << 16);
        d[1] = __uint_as_float(u & 0xffff0000u);
    }
    static __device__ __forceinline__ void store(float *p, const float (&x)[2]) {
        typedef float f2 __attribute__((ext_vector_type(2)));
        __builtin_nontemporal_store((f2){x[0], x[1]}, reinterpret_cast<f2 *>(p));
    }
};
template <> struct ColVec<4> {
    template <typename T> static __device__ __forceinline__ void load(const T *p, size_t i, float (&d)[4]) {
        const float4 x = ld4(p, i);
        d[0] = x.x;
        d[1] = x.y;
        d[2] = x.z;
        d[3] = x.w;
    }
    static __device__ __forceinline__ void store(float *p, const float (&x)[4]) {
        store4_streaming(p, make_float4(x[0], x[1], x[2], x[3]));
    }
};

template <typename T, int RT, int CPL>
struct ContextPhase {
    static constexpr int KB = CPL == 4 ? 8 : FW_KB;     // value rows per batch (two batches in flight per wave)
    static constexpr int NR4 = RT / 4;
    typedef RowPiece<T, CPL> Piece;
    Piece vcur[KB], vnxt[KB];

    // rows kb0 .. kb0 + KB - 1 of column group g.  Buffer loads (lane column as vector offset, row as scalar offset):
    // with a 64-bit address per lane and load the compiler recycled the address registers and made every batch wait
    // for the one before it, so that only one batch was ever under way.
    __device__ __forceinline__ void fetch(Piece (&dst)[KB], const T *vb, int Dv, int L, int lane, int g, int kb0) {
        const BufferRows<T> rows(vb, (unsigned)L * (unsigned)Dv);
        const unsigned col = (unsigned)min((g * 64 + lane) * CPL, Dv - CPL) * (unsigned)sizeof(T);
        const unsigned pitch = (unsigned)Dv * (unsigned)sizeof(T);
#pragma unroll
        for (int kk = 0; kk < KB; ++kk) dst[kk].load(rows, col, (unsigned)min(kb0 + kk, L - 1) * pitch);
    }
    __device__ __forceinline__ void start(const T *vb, int Dv, int L, int lane, int w) {
        const int n_grp = (Dv + 64 * CPL - 1) / (64 * CPL);
        fetch(vcur, vb, Dv, L, lane, min(w, n_grp - 1), 0);
    }
    __device__ __forceinline__ void run(const T *vb, const float *s_S, int spitch, float *Cb, int Dv, int L, int Lp,
                                        int ni, int lane, int w, int n_waves) {
        const int n_grp = (Dv + 64 * CPL - 1) / (64 * CPL);
        const int lr = lane & 3;
        f32x4 acc[CPL][NR4];
#pragma unroll
        for (int c = 0; c < CPL; ++c)
#pragma unroll
            for (int t = 0; t < NR4; ++t) acc[c][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
        int g = w, kb0 = 0;
        // one batch of value rows: products of `cur`, whose successor goes into `nxt` meanwhile; the two register
        // groups change roles from batch to batch (no copies)
        auto batch = [&](Piece (&cur)[KB], Piece (&nxt)[KB]) {
            int g2 = g, kb2 = kb0 + KB;
            if (kb2 >= Lp) {
                g2 = g + n_waves;
                kb2 = 0;
            }
            fetch(nxt, vb, Dv, L, lane, min(g2, n_grp - 1), kb2);
#pragma unroll
            for (int kk = 0; kk < KB; ++kk) cur[kk].pin();
#pragma unroll
            for (int k4 = 0; k4 < KB; k4 += 4) {
                if (kb0 + k4 < Lp) {
                    float4 pr[NR4];
#pragma unroll
                    for (int t = 0; t < NR4; ++t)
                        pr[t] = *reinterpret_cast<const float4 *>(s_S + (4 * t + lr) * spitch + kb0 + k4);
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int c = 0; c < CPL; ++c)
#pragma unroll
                            for (int t = 0; t < NR4; ++t)
                                acc[c][t] = __builtin_amdgcn_mfma_f32_4x4x1f32(comp(pr[t], q), cur[k4 + q].value(c),
                                                                               acc[c][t], 0, 0, 0);
                }
            }
            if (kb2 == 0) {                                        // last batch of column group g
                const int n = (g * 64 + lane) * CPL;
                if (n < Dv) {
#pragma unroll
                    for (int t = 0; t < NR4; ++t)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (4 * t + r < ni) {
                                float x[CPL];
#pragma unroll
                                for (int c = 0; c < CPL; ++c) x[c] = acc[c][t][r];
                                ColVec<CPL>::store(&Cb[(size_t)(4 * t + r) * Dv + n], x);
                            }
                }
#pragma unroll
                for (int c = 0; c < CPL; ++c)
#pragma unroll
                    for (int t = 0; t < NR4; ++t) acc[c][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
            }
            g = g2;
            kb0 = kb2;
        };
        while (g < n_grp) {
            batch(vcur, vnxt);
            if (g >= n_grp) break;
            batch(vnxt, vcur);
        }
    }
};

// The context phase when at least half of the waves would have no columns (value rows of 256 columns per wave, eight
// waves, Dv = 1024): two waves share a column group and take half of the keys each, so that all waves have loads under
// way; the second wave's partial tile reaches the first through LDS (s_x: RT x Dv floats that nobody reads any more, the
// staged query rows), which adds it and writes the context rows.
template <typename T, int RT>
struct ContextSplitKeys {
    static constexpr int CPL = 4, KB = 8, NR4 = RT / 4;
    typedef RowPiece<T, CPL> Piece;
    Piece vcur[KB], vnxt[KB];
    int g, half, k0, k1;                // column group, which half of the keys, keys k0 .. k1 - 1 (multiples of 4)

    __device__ __forceinline__ void fetch(Piece (&dst)[KB], const T *vb, int Dv, int L, int lane, int kb0) {
        const BufferRows<T> rows(vb, (unsigned)L * (unsigned)Dv);
        const unsigned col = (unsigned)min((g * 64 + lane) * CPL, Dv - CPL) * (unsigned)sizeof(T);
        const unsigned pitch = (unsigned)Dv * (unsigned)sizeof(T);
#pragma unroll
        for (int kk = 0; kk < KB; ++kk) dst[kk].load(rows, col, (unsigned)min(kb0 + kk, L - 1) * pitch);
    }
    __device__ __forceinline__ void start(const T *vb, int Dv, int L, int Lp, int lane, int w) {
        const int n_grp = (Dv + 64 * CPL - 1) / (64 * CPL);
        g = w % n_grp;
        half = w / n_grp;
        const int Lh = ((Lp / 4 + 1) / 2) * 4;
        k0 = half == 0 ? 0 : half == 1 ? Lh : Lp;                // waves past the second half (if any) have no keys
        k1 = half == 0 ? Lh : Lp;
        if (k0 < k1) fetch(vcur, vb, Dv, L, lane, k0);
    }
    __device__ __forceinline__ void run(const T *vb, const float *s_S, int spitch, float *s_x, float *Cb, int Dv, int L,
                                        int ni, int lane) {
        const int lr = lane & 3;
        f32x4 acc[CPL][NR4];
#pragma unroll
        for (int c = 0; c < CPL; ++c)
#pragma unroll
            for (int t = 0; t < NR4; ++t) acc[c][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
        int kb0 = k0;
        auto batch = [&](Piece (&cur)[KB], Piece (&nxt)[KB]) {
            if (kb0 + KB < k1) fetch(nxt, vb, Dv, L, lane, kb0 + KB);
#pragma unroll
            for (int kk = 0; kk < KB; ++kk) cur[kk].pin();
#pragma unroll
            for (int k4 = 0; k4 < KB; k4 += 4) {
                if (kb0 + k4 < k1) {
                    float4 pr[NR4];
#pragma unroll
                    for (int t = 0; t < NR4; ++t)
                        pr[t] = *reinterpret_cast<const float4 *>(s_S + (4 * t + lr) * spitch + kb0 + k4);
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int c = 0; c < CPL; ++c)
#pragma unroll
                            for (int t = 0; t < NR4; ++t)
                                acc[c][t] = __builtin_amdgcn_mfma_f32_4x4x1f32(comp(pr[t], q), cur[k4 + q].value(c),
                                                                               acc[c][t], 0, 0, 0);
                }
            }
            kb0 += KB;
        };
        while (kb0 < k1) {
            batch(vcur, vnxt);
            if (kb0 >= k1) break;
            batch(vnxt, vcur);
        }
        const int n = (g * 64 + lane) * CPL;                      // < Dv: every group is whole in this form
        if (half == 1) {
#pragma unroll
            for (int t = 0; t < NR4; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    *reinterpret_cast<float4 *>(s_x + (4 * t + r) * Dv + n) =
                        make_float4(acc[0][t][r], acc[1][t][r], acc[2][t][r], acc[3][t][r]);
        }
        lds_barrier();
        if (half == 0) {
#pragma unroll
            for (int t = 0; t < NR4; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (4 * t + r < ni) {
                        const float4 o = *reinterpret_cast<const float4 *>(s_x + (4 * t + r) * Dv + n);
                        const float x[CPL] = {acc[0][t][r] + o.x, acc[1][t][r] + o.y, acc[2][t][r] + o.z,
                                              acc[3][t][r] + o.w};
                        ColVec<CPL>::store(&Cb[(size_t)(4 * t + r) * Dv + n], x);
                    }
        }
    }
};

// The context phase for short key axes (at most 64 keys) and at most one group of 64 columns per wave: a lane owns
// one column and requests ALL value rows of it at once, before the softmax, so that they arrive while the block waits
// for its last scores and normalises them; the products then find their operands in registers.  (With batches of
// 16 rows one ahead every further batch was a trip to memory that the 32 products of the batch before could not
// cover: 1.4 us for a block with 16 keys, 3.1 us for one with 50.)
template <typename T, int RT>
struct ContextAllRows {
    static constexpr int NR4 = RT / 4;
    typename BufferRows<T>::Raw v[4][16];
    __device__ __forceinline__ void start(const T *vb, int Dv, int L, int lane, int w) {
        const int n = min(w * 64 + lane, Dv - 1);
        const int Lp = (L + 3) & ~3;
        // Buffer loads: the lane's column is the vector offset, the same for all rows, and the row a scalar offset, so
        // nothing is written to vector registers between the loads.  With 64-bit addresses per lane the compiler
        // recycled eight address registers and put waits for the loads already under way in front of every
        // further group of eight: the "all rows at once" took a trip to memory per group.  The descriptor covers the
        // sample's valid rows (the hardware checks the range); rows L .. Lp - 1 repeat the last one.
        const BufferRows<T> rows(vb, (unsigned)L * (unsigned)Dv);
        const unsigned col = (unsigned)n * (unsigned)sizeof(T);
        const unsigned pitch = (unsigned)Dv * (unsigned)sizeof(T);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if (16 * g < Lp) {                                   // uniform; run() reads a group under the same condition
#pragma unroll
                for (int kk = 0; kk < 16; ++kk) v[g][kk] = rows.load_raw(col, (unsigned)min(16 * g + kk, L - 1) * pitch);
            }
        }
    }
    __device__ __forceinline__ void run(const float *s_S, int spitch, float *Cb, int Dv, int Lp, int ni, int lane,
                                        int w) {
        const int n = w * 64 + lane;
        if (w * 64 >= Dv) return;                                // a wave without columns (uniform)
        const int lr = lane & 3;
        f32x4 acc[NR4];
#pragma unroll
        for (int t = 0; t < NR4; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int g = 0; g < 4; ++g) {
#pragma unroll
            for (int k4 = 0; k4 < 16; k4 += 4) {
                if (16 * g + k4 < Lp) {                          // uniform
                    float4 pr[NR4];
#pragma unroll
                    for (int t = 0; t < NR4; ++t)
                        pr[t] = *reinterpret_cast<const float4 *>(s_S + (4 * t + lr) * spitch + 16 * g + k4);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float vq = BufferRows<T>::value(v[g][k4 + q]);
#pragma unroll
                        for (int t = 0; t < NR4; ++t)
                            acc[t] = __builtin_amdgcn_mfma_f32_4x4x1f32(comp(pr[t], q), vq, acc[t], 0, 0, 0);
                    }
                }
            }
        }
        if (n < Dv) {
#pragma unroll
            for (int t = 0; t < NR4; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (4 * t + r < ni) store_streaming(&Cb[(size_t)(4 * t + r) * Dv + n], acc[t][r]);
        }
    }
};

// Which (sample, row tile) this block works on and the sample's valid keys; see "Placement" at the top.
// Ranked mode: wave 0 finds the sample that holds a given rank by radix selection over composite keys
// (valid keys, then index) held two per lane, and hands the answer to the other waves through s_pick.
// Returns false if the block has nothing to do (uniformly for the whole block).
__device__ __forceinline__ bool fw_pick_item(const int *__restrict__ key_len, int B, int Tk, int tiles, int ranked,
                                             int *s_pick, int &b, int &tile, int &L) {
    const int xcd = blockIdx.x % FW_XCD, li = blockIdx.x / FW_XCD;
    if (!ranked) {                         // samples x, x+8, ... on XCD x, in index order
        b = xcd + FW_XCD * (li / tiles);
        tile = li % tiles;
        if (b >= B) return false;
        L = clamp_len(key_len[b], Tk);
        return true;
    }
    // samples of this XCD: ranks 16 g + xcd and 16 g + 15 - xcd (snake over the XCDs), heaviest first
    const int rem = B % (2 * FW_XCD);
    const int M = 2 * (B / (2 * FW_XCD)) + (xcd < rem ? 1 : 0) + (2 * FW_XCD - 1 - xcd < rem ? 1 : 0);
    const int n = M * tiles;               // tiles of this XCD
    if (li >= n) return false;
    // position in the launch order -> position in "heaviest first" order
    int rho = li;
    if (n > FW_CU_PER_XCD && n <= 2 * FW_CU_PER_XCD) {
        const int singles = 2 * FW_CU_PER_XCD - n;             // CUs that get one block: the heaviest tiles
        if (li >= FW_CU_PER_XCD) rho = n - 1 - (li - FW_CU_PER_XCD);
        else if (li >= FW_CU_PER_XCD - singles) rho = li - (FW_CU_PER_XCD - singles);
        else rho = singles + li;
    }
    const int m = rho / tiles;             // the tiles of a sample weigh the same
    tile = rho % tiles;
    if (wave_id() == 0) {
        const int lane = lane_id();
        const int c0 = lane, c1 = lane + 64;
        // larger key = more valid keys, ties to the lower index; bits: length above 7 bits of (127 - index)
        // both counts are requested before either is used (as two guarded loads the second left only after the
        // first had arrived: a second trip to memory for batches of more than 64)
        const int len0 = key_len[min(c0, B - 1)], len1 = key_len[min(c1, B - 1)];
        const unsigned key0 = c0 < B ? ((unsigned)clamp_len(len0, Tk) << 7) | (unsigned)(127 - c0) : 0u;
        const unsigned key1 = c1 < B ? ((unsigned)clamp_len(len1, Tk) << 7) | (unsigned)(127 - c1) : 0u;
        unsigned long long act0 = __ballot(c0 < B), act1 = __ballot(c1 < B);
        int r = (m / 2) * (2 * FW_XCD) + ((m & 1) ? 2 * FW_XCD - 1 - xcd : xcd);   // keys larger than the wanted one
        const int top = 7 + 32 - __builtin_clz((unsigned)Tk);                        // bits in use
        for (int bit = top - 1; bit >= 0; --bit) {
            const unsigned long long m0 = __ballot((key0 >> bit) & 1u) & act0;
            const unsigned long long m1 = __ballot((key1 >> bit) & 1u) & act1;
            const int cnt = __popcll(m0) + __popcll(m1);
            if (cnt > r) {
                act0 = m0;
                act1 = m1;
            } else {
                r -= cnt;
                act0 &= ~m0;
                act1 &= ~m1;
            }
        }
        // exactly one candidate is left
        const bool mine = act0 ? ((act0 >> lane) & 1ull) != 0 : ((act1 >> lane) & 1ull) != 0;
        if (mine) {
            s_pick[0] = act0 ? c0 : c1;
            s_pick[1] = (int)((act0 ? key0 : key1) >> 7);
        }
    }
    lds_barrier();
    b = s_pick[0];
    L = s_pick[1];
    return true;
}

// items dealt to the W waves of a block as contiguous ranges: first item of wave w (w = W gives n)
template <int W> __device__ __forceinline__ int deal_begin(int n, int w) {
    if constexpr (W == 8) return deal8_begin(n, w);
    else return (int)((unsigned)(n * w) / (unsigned)W);
}

template <typename T, int NG, int ROWNS, int W>
__global__ __launch_bounds__(64 * W, NG == 1 ? 4 : 2) void k_fwd_fused(
    const T *__restrict__ Qp, const T *__restrict__ Kp, const T *__restrict__ V, const T *__restrict__ v,
    const int *__restrict__ key_len, float *__restrict__ C, float *__restrict__ P,
    int B, int Tq, int Tk, int H, int Dv, int tiles, int rows_base, int Hp, int spitch, int ranked) {
    constexpr int RT = 8 * NG;
    constexpr int FW_THREADS = 64 * W;
    constexpr int NB = 32 / W;                                 // 16-byte pieces per thread and staging batch
    constexpr bool ROWMODE = ROWNS > 0;                       // ROWNS: slices of h in row mode, 0 = streaming mode
    constexpr int NKM = fw_row_max_keys(ROWNS);
    extern __shared__ __align__(16) float smem[];
    float *s_e = smem;                       // [RT][Hp]  exp(2q) / v
    float *s_c = s_e + RT * Hp;              // [Hp]      1 / v
    float *s_S = s_c + Hp;                   // [RT][spitch]  scores, then probabilities
    __shared__ float s_red[2 * W];

    const int lane = lane_id(), w = wave_id();
    // Two blocks share a CU and reach their phases at different times.  The short phases that wait on memory
    // (placement, staging, softmax, context) go first when they have something to issue; the long score loop
    // of the other block fills the remaining slots.  Without this a block that is still staging gets almost
    // no issue slots while its neighbour is in the score loop.
    __builtin_amdgcn_s_setprio(3);

    // v does not depend on the placement: the first batch of its loads leaves before the key counts are read
    // (in wave 0, which reads the key counts and must not queue them behind anything, right after that)
    // The row tile as pieces of 64 lanes x 16 bytes: piece m is slice m % ns of row m / ns; wave w takes pieces
    // w, w + W, ...  The piece numbers are the same in all lanes, and m * ceil(2^16 / ns) >> 16 = m / ns as long as
    // m ns < 2^16, so that rows and columns cost scalar multiplications (a division per piece, which is what
    // `e / q4` on the thread's element number compiled to, was most of the instructions of this phase).
    const int ns = Hp / FW_SS, n_pc = RT * ns;
    const int ns_inv = __builtin_amdgcn_readfirstlane((65536 + ns - 1) / ns);
    auto piece_row = [&](int m) { return (m * ns_inv) >> 16; };
    auto piece_col = [&](int m, int a) { return (m - a * ns) * FW_SS + 4 * lane; };
    // (v and the query rows stay as loaded until the staging loop: see RawKey)
    RawKey<T> vv[NB];
    auto load_v = [&]() {
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int m = w + u * W;
            const int h = piece_col(m, piece_row(m));
            if (m < n_pc && h < H) vv[u].load(v, (size_t)h);
            else vv[u].zero();
        }
    };
    if (w != 0) load_v();

    __shared__ int s_pick[2];
    int b, tile, L;
    if (!fw_pick_item(key_len, B, Tk, tiles, ranked, s_pick, b, tile, L)) return;
    if (w == 0) load_v();
    b = __builtin_amdgcn_readfirstlane(b);
    tile = __builtin_amdgcn_readfirstlane(tile);
    L = __builtin_amdgcn_readfirstlane(L);
    // rows are split evenly over the tiles: rows_base = Tq / tiles each (from the host: a division here is a long
    // subroutine on the vector unit in every wave), the first Tq % tiles of them one more
    const int rows_extra = Tq - rows_base * tiles;
    const int r0 = tile * rows_base + min(tile, rows_extra);
    const int ni = rows_base + (tile < rows_extra ? 1 : 0);   // 1..RT

    float *Pb = P + ((size_t)b * Tq + r0) * Tk;
    float *Cb = C + ((size_t)b * Tq + r0) * Dv;
    if (L == 0) {                                             // no valid key: zeros
        for (int e = threadIdx.x; e < ni * Tk; e += FW_THREADS) Pb[e] = 0.f;
        for (int e = threadIdx.x; e < ni * Dv; e += FW_THREADS) Cb[e] = 0.f;
        return;
    }

    // ---- loads first, in the order of their use: the first batch of query rows (four 16-byte loads per
    // thread; v was requested before the placement), then this wave's keys (row mode: all of them, streaming
    // mode: the first slice); then A: exp(2q)/v and 1/v to LDS (rows past ni and columns past H: 0 and kHugeC)
    const T *qb = Qp + ((size_t)b * Tq + r0) * H;
    const T *kb = Kp + (size_t)b * Tk * H;
    RawKey<T> x[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
        const int m = w + u * W;
        const int a = piece_row(m), h = piece_col(m, a);
        if (m < n_pc && h < H && a < ni) x[u].load(qb + (size_t)a * H, (size_t)h);
        else x[u].zero();
    }
    const int k_lo = deal_begin<W>(L, w);
    const int nk = deal_begin<W>(L, w + 1) - k_lo;
    KeyStream<T> ks;
    RawKey<T> raw[ROWMODE ? ROWNS : 1][NKM];
    if constexpr (ROWMODE) {
        // only the wave's own keys are requested (every load takes its turn in the CU's address unit whether
        // it hits or not); the branches are uniform and everything is awaited at the staging barrier anyway
#pragma unroll
        for (int c = 0; c < NKM; ++c) {
            if (c < nk) {
#pragma unroll
                for (int s = 0; s < ROWNS; ++s) {
                    const int hc = min(s * FW_SS + 4 * lane, H - 4);   // columns past H: see KeyStream::fetch
                    raw[s][c].load(kb, (size_t)(unsigned)((k_lo + c) * H + hc));
                }
            } else {
#pragma unroll
                for (int s = 0; s < ROWNS; ++s) raw[s][c].zero();
            }
        }
    } else {
        ks.init(kb, H, lane, k_lo, nk, Hp / FW_SS);
        ks.start();
    }

    float qe_m = 0.f, c_m = 0.f;
    for (int m0 = w; m0 < n_pc; m0 += NB * W) {
        if (m0 != w) {                                         // later batches (H > 1024): loaded here
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const int m = m0 + u * W;
                const int a = piece_row(m), h = piece_col(m, a);
                const bool in = m < n_pc && h < H;
                if (in && a < ni) x[u].load(qb + (size_t)a * H, (size_t)h);
                else x[u].zero();
                if (in) vv[u].load(v, (size_t)h);
                else vv[u].zero();
            }
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            x[u].pin();
            vv[u].pin();
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int m = m0 + u * W;
            if (m < n_pc) {
                const int a = piece_row(m), h = piece_col(m, a);
                const bool row_on = a < ni;
                const float4 x4 = x[u].get(), v4 = vv[u].get();
                float y[4], cc[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float vq = comp(v4, q);
                    const bool v_on = fabsf(vq) >= kTinyV;         // false for columns past H (v read as 0)
                    cc[q] = v_on ? fast_rcp(vq) : kHugeC;
                    y[q] = (v_on && row_on) ? fast_exp2(kTwoLog2e * comp(x4, q)) * cc[q] : 0.f;
                    qe_m = fmaxf(qe_m, fabsf(y[q]));
                    // a |v| so large that products of two 1/v could underflow also goes to the exact path
                    c_m = fmaxf(c_m, fabsf(vq) > 1e15f ? INFINITY : fabsf(cc[q]));
                    if (y[q] != y[q]) qe_m = INFINITY;              // NaN input: exact path (fmaxf drops NaN)
                }
                *reinterpret_cast<float4 *>(s_e + a * Hp + h) = make_float4(y[0], y[1], y[2], y[3]);
                if (a == 0) *reinterpret_cast<float4 *>(s_c + h) = make_float4(cc[0], cc[1], cc[2], cc[3]);
            }
        }
    }
    qe_m = wave_max(qe_m);
    c_m = wave_max(c_m);
    if (lane == 0) {
        s_red[w] = qe_m;
        s_red[W + w] = c_m;
    }
    lds_barrier();
    float qe_max = 0.f, c_max = 0.f;
#pragma unroll
    for (int k = 0; k < W; ++k) {
        qe_max = fmaxf(qe_max, s_red[k]);
        c_max = fmaxf(c_max, s_red[W + k]);
    }

    // ---- B: scores of this wave's keys
    __builtin_amdgcn_s_setprio(0);
    if constexpr (ROWMODE) {
        // the keys are used from here on (see RawKey)
#pragma unroll
        for (int s = 0; s < ROWNS; ++s)
#pragma unroll
            for (int c = 0; c < NKM; ++c) raw[s][c].pin();
        if (fw_rows_n<T, ROWNS, NKM>(nk, raw, s_e, s_c, Hp, ni, qe_max, c_max, s_S, spitch, k_lo))
            fw_pass_exact<T>(qb, ni, kb + (size_t)k_lo * H, nk, H, v, s_S, spitch, k_lo);
    } else {
        for (int p = 0; p < ks.npass; ++p) {                   // passes of up to FW_NJ keys
            const int j0 = ks.pass_begin(p);
            const int nj = ks.pass_begin(p + 1) - j0;          // 1..FW_NJ
            bool redo = true;
#define FW_CASE(N)                                                                                          \
    case N:                                                                                                 \
        redo = (ni == RT)       ? fw_pass<T, NG, N, RT>(s_e, s_c, Hp, ni, ks, qe_max, c_max, s_S, spitch, j0)     \
               : (ni == RT - 1) ? fw_pass<T, NG, N, RT - 1>(s_e, s_c, Hp, ni, ks, qe_max, c_max, s_S, spitch, j0) \
                                : fw_pass<T, NG, N, 0>(s_e, s_c, Hp, ni, ks, qe_max, c_max, s_S, spitch, j0);     \
        break;
            switch (nj) {
                FW_CASE(1) FW_CASE(2) FW_CASE(3) FW_CASE(4)
                default: break;
            }
#undef FW_CASE
            if (redo) fw_pass_exact<T>(qb, ni, kb + (size_t)j0 * H, nj, H, v, s_S, spitch, j0);
        }
    }
    __builtin_amdgcn_s_setprio(3);

    // ---- C and D: softmax, then context rows = P V; the first batch of value rows leaves before the softmax.
    // Wide value rows take two or four columns per lane (8- or 16-byte loads).
    const T *vb = V + (size_t)b * Tk * Dv;
    const int Lp = (L + 3) & ~3;
    auto softmax = [&]() {
        lds_barrier();
        // waves take rows in turn; probabilities replace the scores in LDS
        for (int a = w; a < RT; a += W) {
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
                    if (j < Tk) store_streaming(&Pb[(size_t)a * Tk + j], p);
                }
            } else {
                for (int j = lane; j < Lp; j += 64) srow[j] = 0.f;
            }
        }
        lds_barrier();
    };
    if (ROWMODE && Tk <= 64 && Dv <= 64 * W) {                  // all value rows of a wave's columns at once
        ContextAllRows<T, RT> cp;
        cp.start(vb, Dv, L, lane, w);
        softmax();
        cp.run(s_S, spitch, Cb, Dv, Lp, ni, lane, w);
    } else if (Dv % 256 == 0 && 2 * (Dv / 256) == W && Dv <= Hp) {   // two waves per group of 256 columns
        ContextSplitKeys<T, RT> cp;
        cp.start(vb, Dv, L, Lp, lane, w);
        softmax();
        cp.run(vb, s_S, spitch, s_e, Cb, Dv, L, ni, lane);
    } else if (Dv >= 1024) {                                    // at least four waves with columns to work on
        ContextPhase<T, RT, 4> cp;
        cp.start(vb, Dv, L, lane, w);
        softmax();
        cp.run(vb, s_S, spitch, Cb, Dv, L, Lp, ni, lane, w, W);
    } else if (Dv >= 512) {
        ContextPhase<T, RT, 2> cp;
        cp.start(vb, Dv, L, lane, w);
        softmax();
        cp.run(vb, s_S, spitch, Cb, Dv, L, Lp, ni, lane, w, W);
    } else {
        ContextPhase<T, RT, 1> cp;
        cp.start(vb, Dv, L, lane, w);
        softmax();
        cp.run(vb, s_S, spitch, Cb, Dv, L, Lp, ni, lane, w, W);
    }
}


// Rows per block: 8.  (16 rows halve the exponentials of K per score, but need twice the accumulators; with
// two waves per SIMD instead of four that measured 20-25 % slower on the large workloads.)

static size_t fwd_lds_bytes(const AttnShape &s, int ng) {
    const int Hp = (s.H + FW_SS - 1) / FW_SS * FW_SS;
    const int spitch = ((s.Tk + 3) & ~3) + 4;
    return ((size_t)(8 * ng) * (Hp + spitch) + Hp) * sizeof(float);
}

bool fwd_fused_supported(const AttnShape &s) {
    // the context phase addresses a sample's value rows by 32-bit byte offsets (BufferRows)
    const bool v_in_range = (long long)s.Tk * s.Dv * (s.bf16 ? 2 : 4) < (1LL << 31);
    return s.H % 4 == 0 && fwd_lds_bytes(s, 1) <= 150 * 1024 && v_in_range;
}

// Row mode needs the longest key share of a wave, ceil(Tk / 8) keys, times the slices of h to fit the
// registers set aside for it; it is built for 1, 2 and 4 slices (H up to 256, 512, 1024).
static int fwd_row_mode_slices(const AttnShape &s) {
    const int ns = (s.H + FW_SS - 1) / FW_SS;
    if (ns != 1 && ns != 2 && ns != 4) return 0;
    return (s.Tk + FW_W - 1) / FW_W <= fw_row_max_keys(ns) ? ns : 0;
}

template <typename T, int NG, int ROWNS, int W>
static hipError_t launch_fwd_fused_t(const AttnShape &s, const void *Qp, const void *Kp, const void *V, const void *v,
                                     const int *key_len, float *C, float *P, hipStream_t st) {
    constexpr int RT = 8 * NG;
    const int Hp = (s.H + FW_SS - 1) / FW_SS * FW_SS;
    const int spitch = ((s.Tk + 3) & ~3) + 4;
    const size_t lds = fwd_lds_bytes(s, NG);
    if (lds > 48 * 1024) {   // beyond the default dynamic LDS limit
        static LdsGrants granted;
        hipError_t e = ensure_dynamic_lds((const void *)k_fwd_fused<T, NG, ROWNS, W>, lds, granted);
        if (e != hipSuccess) return e;
    }
    int tiles = (s.Tq + RT - 1) / RT;
    const int samples_per_xcd = (s.B + FW_XCD - 1) / FW_XCD;
    // Row mode with less than one round of blocks (two per CU): more, smaller row tiles while the grid still fits
    // the round, so that every CU holds a heavy and a light tile (with 448 blocks 64 CUs held a single heavy one and
    // the fullest CU 18 % more keys than the average; with 512 it is 5 %; the keys are exponentiated once more per sample).
    // At most twice the tiles (at least RT / 2 rows each).
    // (Streaming mode loses with smaller tiles: 74 -> 82 us at B = 128, T = 100, where whole rounds were filled that way.)
    if (ROWNS > 0 && W == FW_W) {
        const int most = min(s.Tq, 2 * tiles);
        while (tiles < most && (long long)FW_XCD * samples_per_xcd * (tiles + 1) <= 2 * FW_XCD * FW_CU_PER_XCD) ++tiles;
    }
    const long long grid = (long long)FW_XCD * samples_per_xcd * tiles;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    const int ranked = s.B <= FW_MAX_RANKED_B ? 1 : 0;
    k_fwd_fused<T, NG, ROWNS, W><<<(unsigned)grid, 64 * W, lds, st>>>(
        (const T *)Qp, (const T *)Kp, (const T *)V, (const T *)v, key_len, C, P, s.B, s.Tq, s.Tk, s.H, s.Dv, tiles,
        s.Tq / tiles, Hp, spitch, ranked);
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_fwd_fused_mode(const AttnShape &s, const void *Qp, const void *Kp, const void *V,
                                        const void *v, const int *key_len, float *C, float *P, hipStream_t st) {
    switch (fwd_row_mode_slices(s)) {
        case 1: return launch_fwd_fused_t<T, 1, 1, FW_W>(s, Qp, Kp, V, v, key_len, C, P, st);
        case 2: return launch_fwd_fused_t<T, 1, 2, FW_W>(s, Qp, Kp, V, v, key_len, C, P, st);
        case 4: return launch_fwd_fused_t<T, 1, 4, FW_W>(s, Qp, Kp, V, v, key_len, C, P, st);
        default: break;
    }
    // Streaming mode.  Up to two slices of h (H <= 512): blocks of four waves, four of them on a CU (measured 9 %
    // faster at B = 128, T = 100, H = 512); beyond that the row tile's LDS allows only three such blocks and the
    // eight-wave block, two per CU, keeps more waves resident (four-wave blocks measured 2 % slower at H = 1024).
    if (s.H <= 2 * FW_SS) return launch_fwd_fused_t<T, 1, 0, FW_W_STREAM>(s, Qp, Kp, V, v, key_len, C, P, st);
    return launch_fwd_fused_t<T, 1, 0, FW_W>(s, Qp, Kp, V, v, key_len, C, P, st);
}

hipError_t launch_fwd_fused(const AttnShape &s, const void *Qp, const void *Kp, const void *V, const void *v,
                            const int *key_len, float *C, float *P, hipStream_t st) {
    return s.bf16 ? launch_fwd_fused_mode<bf16_t>(s, Qp, Kp, V, v, key_len, C, P, st)
                  : launch_fwd_fused_mode<float>(s, Qp, Kp, V, v, key_len, C, P, st);
}

}  // namespace echo
