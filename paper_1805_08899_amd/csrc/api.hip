// C ABI of libechoattn: argument validation, workspace carving and the
// sequence of kernel launches.  No allocation, no synchronisation.
#include "../../include/echoattn.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <mutex>
#include <string>
#include <vector>

#include "kernels.hpp"

namespace {

using echo::AttnShape;

constexpr int kMaxTk = ECHO_ATTN_MAX_TK;            // dP rows of 16 queries live in LDS in the softmax-backward kernel
constexpr int kMaxTkStep = ECHO_ATTN_STEP_MAX_TK;   // one row of scores and one of dS live in LDS in the step kernels
constexpr int kMaxB = ECHO_ATTN_MAX_B;              // the batch is a grid y dimension

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

echo_status_t check_desc(const echo_attn_desc_t *d, AttnShape *s, int max_tk = kMaxTk) {
    if (!d) return ECHO_ERR_NULL;
    if (d->in_dtype != ECHO_F32 && d->in_dtype != ECHO_BF16) return ECHO_ERR_DTYPE;
    if (d->B < 1 || d->Tq < 1 || d->Tk < 1 || d->H < 1 || d->Dv < 1) return ECHO_ERR_SHAPE;
    if (d->Dv % 4 != 0) return ECHO_ERR_SHAPE;            // value rows are read 16 bytes at a time
    if (d->Tk > max_tk) return ECHO_ERR_SHAPE;
    if (d->B > kMaxB) return ECHO_ERR_SHAPE;
    const int64_t lim = (int64_t)1 << 31;
    const int64_t per_sample[] = {(int64_t)d->Tq * d->H, (int64_t)d->Tk * d->H, (int64_t)d->Tk * d->Dv,
                                  (int64_t)d->Tq * d->Dv, (int64_t)d->Tq * (d->Tk + 16)};
    for (int64_t e : per_sample)
        if (e >= lim) return ECHO_ERR_SHAPE;
    // the 4-D map index B*Tq*Tk*H must fit 62 bits (it always does once the lines above hold; kept explicit)
    const long double n4 = (long double)d->B * d->Tq * d->Tk * d->H;
    if (n4 >= 4.6e18L) return ECHO_ERR_SHAPE;
    if (s) *s = AttnShape{d->B, d->Tq, d->Tk, d->H, d->Dv, d->in_dtype == ECHO_BF16, false};
    return ECHO_OK;
}

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

struct BwdWs {
    size_t ds_off, rowsum_off, dvpart_off, order_off, dvflag_off, total;
};
BwdWs bwd_layout(const AttnShape &s) {
    BwdWs w;
    w.ds_off = 0;
    w.rowsum_off = align_up((size_t)s.B * s.Tq * echo::ds_pitch(s.Tk) * sizeof(float));
    w.dvpart_off = w.rowsum_off + align_up((size_t)s.B * s.Tq * sizeof(float));
    w.order_off = w.dvpart_off + align_up((size_t)s.B * s.H * sizeof(float));
    w.dvflag_off = w.order_off + align_up((size_t)s.B * sizeof(int));
    w.total = w.dvflag_off + align_up((size_t)((s.H + 63) / 64) * s.B * sizeof(unsigned long long));
    return w;
}
// scores S [B,Tq,Tk] of the unfused forward kernels; the fused kernel keeps them in LDS and needs nothing
size_t fwd_bytes(const AttnShape &s, bool want_map) {
    if (!want_map && s.Tq == 1 && echo::step_split_mail_bytes(s) > 0) return align_up(echo::step_split_mail_bytes(s));
    if (!want_map && echo::fwd_fused_supported(s)) return 0;
    return align_up((size_t)s.B * s.Tq * s.Tk * sizeof(float));
}

// ---- optional per-kernel timing ------------------------------------------------
struct ProfRec {
    const char *name;
    hipEvent_t t0, t1;
};
thread_local bool g_prof_on = false;
thread_local std::vector<ProfRec> g_prof;

struct Timed {
    const char *name;
    hipStream_t st;
    hipEvent_t t0 = nullptr, t1 = nullptr;
    Timed(const char *n, hipStream_t s) : name(n), st(s) {
        if (g_prof_on && hipEventCreate(&t0) == hipSuccess && hipEventCreate(&t1) == hipSuccess)
            (void)hipEventRecord(t0, st);
    }
    ~Timed() {
        if (t0 && t1) {
            (void)hipEventRecord(t1, st);
            g_prof.push_back({name, t0, t1});
        }
    }
};

thread_local std::string g_last_error;

// Number of a backward launch: blocks of one launch recognise each other's flags in the workspace by it, so
// the flags need no clearing beforehand, whatever the workspace holds.  Odd, hence never 0 (the cleared state).
std::atomic<unsigned long long> g_launch_number{0x9E3779B97F4A7C15ull};
unsigned long long next_launch_number() { return g_launch_number.fetch_add(2, std::memory_order_relaxed) | 1ull; }

// A HIP error left pending on the calling thread by earlier, unrelated calls is cleared first, so that what
// is reported belongs to this launch.
#define ECHO_LAUNCH(NAME, CALL)                                                  \
    do {                                                                         \
        hipError_t e_;                                                           \
        (void)hipGetLastError();                                                 \
        {                                                                        \
            Timed t_(NAME, st);                                                  \
            e_ = (CALL);                                                         \
        }                                                                        \
        if (e_ != hipSuccess) {                                                  \
            g_last_error = std::string(NAME) + ": " + hipGetErrorString(e_);     \
            return ECHO_ERR_HIP;                                                 \
        }                                                                        \
    } while (0)

echo_status_t fwd_impl(const echo_attn_desc_t *desc, const void *Qp, const void *Kp, const void *V, const void *v,
                       const int32_t *key_len, float *context, float *P, float *tmap, bool want_map,
                       void *workspace, size_t workspace_bytes, void *stream) {
    AttnShape s;
    echo_status_t rc = check_desc(desc, &s);
    if (rc != ECHO_OK) return rc;
    const size_t need = fwd_bytes(s, want_map);
    if (!Qp || !Kp || !V || !v || !key_len || !context || !P || (need > 0 && !workspace)) return ECHO_ERR_NULL;
    if (want_map && !tmap) return ECHO_ERR_NULL;
    const void *ptrs[] = {Qp, Kp, V, v, key_len, context, P, workspace, tmap};
    for (const void *p : ptrs)
        if (p && misaligned(p)) return ECHO_ERR_ALIGN;
    if (workspace_bytes < need) return ECHO_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    float *S = static_cast<float *>(workspace);
    if (!want_map && s.Tq == 1) {             // a decoder step: the kernels made for one query per sample
        if (echo::step_split_applicable(s)) {
            ECHO_LAUNCH("step_fwd_split", echo::launch_step_fwd_split(s, Qp, Kp, V, v, key_len, context, P, workspace,
                                                                      next_launch_number(), st));
            return ECHO_OK;
        }
        if (echo::step_lds_bytes(s) <= 64 * 1024) {
            ECHO_LAUNCH("step_fwd", echo::launch_step_fwd(s, Qp, Kp, V, v, key_len, context, P, st));
            return ECHO_OK;
        }
    }
    if (!want_map && echo::fwd_fused_supported(s)) {
        ECHO_LAUNCH("fwd_fused", echo::launch_fwd_fused(s, Qp, Kp, V, v, key_len, context, P, st));
        return ECHO_OK;
    }
    ECHO_LAUNCH(want_map ? "score_stash" : "score",
                echo::launch_score(s, Qp, Kp, v, key_len, S, want_map ? tmap : nullptr, st));
    ECHO_LAUNCH("softmax", echo::launch_softmax(s, S, key_len, P, st));
    ECHO_LAUNCH("context", echo::launch_context(s, P, V, key_len, context, st));
    return ECHO_OK;
}

echo_status_t bwd_impl(const echo_attn_desc_t *desc, const float *dContext, const float *P, const float *tmap,
                       bool use_map, bool accumulate, const void *Qp, const void *Kp, const void *V, const void *v,
                       const int32_t *key_len, float *dQp, float *dKp, float *dV, float *dv, void *workspace,
                       size_t workspace_bytes, void *stream) {
    AttnShape s;
    echo_status_t rc = check_desc(desc, &s);
    if (rc != ECHO_OK) return rc;
    s.acc = accumulate;
    if (!dContext || !P || !V || !v || !key_len || !dQp || !dKp || !dV || !dv || !workspace) return ECHO_ERR_NULL;
    if (use_map ? !tmap : (!Qp || !Kp)) return ECHO_ERR_NULL;
    const void *ptrs[] = {dContext, P, tmap, Qp, Kp, V, v, key_len, dQp, dKp, dV, dv, workspace};
    for (const void *p : ptrs)
        if (p && misaligned(p)) return ECHO_ERR_ALIGN;
    const BwdWs lay = bwd_layout(s);
    if (workspace_bytes < lay.total) return ECHO_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    float *dS = reinterpret_cast<float *>(ws + lay.ds_off);
    float *rowsum = reinterpret_cast<float *>(ws + lay.rowsum_off);
    float *dv_part = reinterpret_cast<float *>(ws + lay.dvpart_off);
    int *order = reinterpret_cast<int *>(ws + lay.order_off);
    unsigned long long *dv_flag = reinterpret_cast<unsigned long long *>(ws + lay.dvflag_off);
    ECHO_LAUNCH("bwd_pre", echo::launch_bwd_pre(s, dContext, V, P, key_len, dS, rowsum, order, dV, st));
    ECHO_LAUNCH(use_map ? "recompute_stash" : "recompute",
                echo::launch_recompute(s, Qp, Kp, v, order, dS, rowsum, use_map ? tmap : nullptr, dQp, dKp, dv_part,
                                       dv_flag, next_launch_number(), dv, st));
    return ECHO_OK;
}

// ---- device memory that belongs to the library: the backward workspace of echo_attn_bwd_static -------------
// In host code `scratch` is only the handle of the symbol, not an address on the device; the address of each
// device's copy is looked up once per device (with that device current) and kept in g_scratch_ptr.
constexpr size_t kStaticScratchBytes = ECHO_ATTN_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

echo_status_t static_scratch(void **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        g_last_error = std::string("static scratch: hipGetDevice: ") + hipGetErrorString(e);
        return ECHO_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            g_last_error = std::string("static scratch: hipGetSymbolAddress: ") + hipGetErrorString(e);
            return ECHO_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ECHO_OK;
}

// The per-sentence buffer of the deferred decoder form: [B, steps, ds_pitch(Tk)] rows of dS, [B, steps] row sums,
// then the mail area of the steps' four-block form (empty where that form does not apply).
AttnShape one_step(AttnShape s) {
    s.Tq = 1;
    return s;
}
size_t steps_mail_offset(const AttnShape &s, int steps) {
    return align_up((size_t)s.B * steps * echo::ds_pitch(s.Tk) * sizeof(float)) + align_up((size_t)s.B * steps * sizeof(float));
}

}  // namespace

extern "C" {

size_t echo_attn_fwd_workspace_bytes(const echo_attn_desc_t *desc) {
    AttnShape s;
    return check_desc(desc, &s) == ECHO_OK ? fwd_bytes(s, false) : 0;
}

size_t echo_attn_bwd_workspace_bytes(const echo_attn_desc_t *desc) {
    AttnShape s;
    return check_desc(desc, &s) == ECHO_OK ? bwd_layout(s).total : 0;
}

size_t echo_attn_fwd_stash_workspace_bytes(const echo_attn_desc_t *desc) {
    AttnShape s;
    return check_desc(desc, &s) == ECHO_OK ? fwd_bytes(s, true) : 0;
}

size_t echo_attn_stash_bytes(const echo_attn_desc_t *desc) {
    AttnShape s;
    if (check_desc(desc, &s) != ECHO_OK) return 0;
    return (size_t)s.B * s.Tq * s.Tk * s.H * sizeof(float);
}

echo_status_t echo_attn_fwd(const echo_attn_desc_t *desc, const void *Qp, const void *Kp, const void *V,
                            const void *v, const int32_t *key_len, float *context, float *P, void *workspace,
                            size_t workspace_bytes, void *stream) {
    return fwd_impl(desc, Qp, Kp, V, v, key_len, context, P, nullptr, false, workspace, workspace_bytes, stream);
}

echo_status_t echo_attn_bwd(const echo_attn_desc_t *desc, const float *dContext, const float *P, const void *Qp,
                            const void *Kp, const void *V, const void *v, const int32_t *key_len, float *dQp,
                            float *dKp, float *dV, float *dv, void *workspace, size_t workspace_bytes,
                            void *stream) {
    return bwd_impl(desc, dContext, P, nullptr, false, false, Qp, Kp, V, v, key_len, dQp, dKp, dV, dv, workspace,
                    workspace_bytes, stream);
}

echo_status_t echo_attn_bwd_static(const echo_attn_desc_t *desc, const float *dContext, const float *P,
                                   const void *Qp, const void *Kp, const void *V, const void *v,
                                   const int32_t *key_len, float *dQp, float *dKp, float *dV, float *dv,
                                   void *stream) {
    AttnShape s;
    echo_status_t rc = check_desc(desc, &s);
    if (rc != ECHO_OK) return rc;
    if (bwd_layout(s).total > kStaticScratchBytes) {
        g_last_error = "echo_attn_bwd_static: this shape needs " + std::to_string(bwd_layout(s).total) +
                       " bytes of workspace, the library's own buffer holds " + std::to_string(kStaticScratchBytes);
        return ECHO_ERR_WORKSPACE;
    }
    void *ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != ECHO_OK) return rc;
    return bwd_impl(desc, dContext, P, nullptr, false, false, Qp, Kp, V, v, key_len, dQp, dKp, dV, dv, ws,
                    kStaticScratchBytes, stream);
}

echo_status_t echo_attn_bwd_accumulate(const echo_attn_desc_t *desc, const float *dContext, const float *P,
                                       const void *Qp, const void *Kp, const void *V, const void *v,
                                       const int32_t *key_len, float *dQp, float *dKp, float *dV, float *dv,
                                       void *workspace, size_t workspace_bytes, void *stream) {
    return bwd_impl(desc, dContext, P, nullptr, false, true, Qp, Kp, V, v, key_len, dQp, dKp, dV, dv, workspace,
                    workspace_bytes, stream);
}

echo_status_t echo_attn_step_fwd(const echo_attn_desc_t *desc, const void *Qp, const void *Kp, const void *V,
                                 const void *v, const int32_t *key_len, float *context, float *P, void *stream) {
    AttnShape s;
    echo_status_t rc = check_desc(desc, &s, kMaxTkStep);
    if (rc != ECHO_OK) return rc;
    if (s.Tq != 1 || echo::step_lds_bytes(s) > 64 * 1024) return ECHO_ERR_SHAPE;
    if (!Qp || !Kp || !V || !v || !key_len || !context || !P) return ECHO_ERR_NULL;
    const void *ptrs[] = {Qp, Kp, V, v, key_len, context, P};
    for (const void *p : ptrs)
        if (misaligned(p)) return ECHO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ECHO_LAUNCH("step_fwd", echo::launch_step_fwd(s, Qp, Kp, V, v, key_len, context, P, st));
    return ECHO_OK;
}

echo_status_t echo_attn_step_bwd(const echo_attn_desc_t *desc, const float *dContext, const float *P,
                                 const void *Qp, const void *Kp, const void *V, const void *v,
                                 const int32_t *key_len, float *dQp, float *dKp, float *dV, float *dv_part,
                                 void *stream) {
    AttnShape s;
    echo_status_t rc = check_desc(desc, &s, kMaxTkStep);
    if (rc != ECHO_OK) return rc;
    if (s.Tq != 1 || echo::step_lds_bytes(s) > 64 * 1024) return ECHO_ERR_SHAPE;
    if (!dContext || !P || !Qp || !Kp || !V || !v || !key_len || !dQp || !dKp || !dV || !dv_part) return ECHO_ERR_NULL;
    const void *ptrs[] = {dContext, P, Qp, Kp, V, v, key_len, dQp, dKp, dV, dv_part};
    for (const void *p : ptrs)
        if (misaligned(p)) return ECHO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ECHO_LAUNCH("step_bwd", echo::launch_step_bwd(s, dContext, P, Qp, Kp, V, v, key_len, dQp, dKp, dV, dv_part, st));
    return ECHO_OK;
}

size_t echo_attn_steps_ds_bytes(const echo_attn_desc_t *desc) {
    AttnShape s;
    if (check_desc(desc, &s) != ECHO_OK) return 0;
    return steps_mail_offset(s, s.Tq) + align_up(echo::step_split_mail_bytes(one_step(s)));
}

echo_status_t echo_attn_step_bwd_query(const echo_attn_desc_t *desc, int32_t step, int32_t steps,
                                       const float *dContext, const float *P, const void *Qp, const void *Kp,
                                       const void *V, const void *v, const int32_t *key_len, float *dQp,
                                       void *ds_rows, void *stream) {
    AttnShape s;
    echo_status_t rc = check_desc(desc, &s);
    if (rc != ECHO_OK) return rc;
    if (s.Tq != 1 || steps < 1 || step < 0 || step >= steps) return ECHO_ERR_SHAPE;
    if ((int64_t)steps * (s.Tk + 16) >= ((int64_t)1 << 31)) return ECHO_ERR_SHAPE;
    if (!dContext || !P || !Qp || !Kp || !V || !v || !key_len || !dQp || !ds_rows) return ECHO_ERR_NULL;
    const void *ptrs[] = {dContext, P, Qp, Kp, V, v, key_len, dQp, ds_rows};
    for (const void *p : ptrs)
        if (misaligned(p)) return ECHO_ERR_ALIGN;
    float *ds = static_cast<float *>(ds_rows);
    float *ds_sum = reinterpret_cast<float *>(static_cast<char *>(ds_rows) +
                                              align_up((size_t)s.B * steps * echo::ds_pitch(s.Tk) * sizeof(float)));
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (echo::step_split_applicable(s)) {
        void *mail = static_cast<char *>(ds_rows) + steps_mail_offset(s, steps);
        ECHO_LAUNCH("step_bwd_query_split",
                    echo::launch_step_bwd_query_split(s, dContext, P, Qp, Kp, V, v, key_len, dQp, ds, ds_sum, steps,
                                                      step, mail, next_launch_number(), st));
        return ECHO_OK;
    }
    ECHO_LAUNCH("step_bwd_query",
                echo::launch_step_bwd_query(s, dContext, P, Qp, Kp, V, v, key_len, dQp, ds, ds_sum, steps, step, st));
    return ECHO_OK;
}

echo_status_t echo_attn_steps_bwd_keys(const echo_attn_desc_t *desc, const float *dContext, const float *P,
                                       const void *Qp, const void *Kp, const void *v, const int32_t *key_len,
                                       const void *ds_rows, float *dKp, float *dV, float *dv, void *workspace,
                                       size_t workspace_bytes, void *stream) {
    AttnShape s;
    echo_status_t rc = check_desc(desc, &s);
    if (rc != ECHO_OK) return rc;
    if (!dContext || !P || !Qp || !Kp || !v || !key_len || !ds_rows || !dKp || !dV || !dv || !workspace) return ECHO_ERR_NULL;
    const void *ptrs[] = {dContext, P, Qp, Kp, v, key_len, ds_rows, dKp, dV, dv, workspace};
    for (const void *p : ptrs)
        if (misaligned(p)) return ECHO_ERR_ALIGN;
    const BwdWs lay = bwd_layout(s);
    if (workspace_bytes < lay.total) return ECHO_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    // dS and its row sums were left by the steps; the call's own workspace holds the rest
    float *dS = const_cast<float *>(static_cast<const float *>(ds_rows));
    float *rowsum = reinterpret_cast<float *>(const_cast<char *>(static_cast<const char *>(ds_rows)) +
                                              align_up((size_t)s.B * s.Tq * echo::ds_pitch(s.Tk) * sizeof(float)));
    float *dv_part = reinterpret_cast<float *>(ws + lay.dvpart_off);
    int *order = reinterpret_cast<int *>(ws + lay.order_off);
    unsigned long long *dv_flag = reinterpret_cast<unsigned long long *>(ws + lay.dvflag_off);
    ECHO_LAUNCH("bwd_pre_dv", echo::launch_bwd_pre(s, dContext, nullptr, P, key_len, dS, rowsum, order, dV, st, false));
    ECHO_LAUNCH("recompute_keys", echo::launch_recompute(s, Qp, Kp, v, order, dS, rowsum, nullptr, nullptr, dKp, dv_part,
                                                         dv_flag, next_launch_number(), dv, st));
    return ECHO_OK;
}

echo_status_t echo_attn_step_finish(const echo_attn_desc_t *desc, const float *dv_part, float *dv, void *stream) {
    AttnShape s;
    echo_status_t rc = check_desc(desc, &s, kMaxTkStep);
    if (rc != ECHO_OK) return rc;
    if (!dv_part || !dv) return ECHO_ERR_NULL;
    if (misaligned(dv_part) || misaligned(dv)) return ECHO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ECHO_LAUNCH("dv_reduce", echo::launch_dv_reduce(s, dv_part, dv, st));
    return ECHO_OK;
}

echo_status_t echo_attn_fwd_stash(const echo_attn_desc_t *desc, const void *Qp, const void *Kp, const void *V,
                                  const void *v, const int32_t *key_len, float *context, float *P,
                                  float *tanh_map, void *workspace, size_t workspace_bytes, void *stream) {
    return fwd_impl(desc, Qp, Kp, V, v, key_len, context, P, tanh_map, true, workspace, workspace_bytes, stream);
}

echo_status_t echo_attn_bwd_stash(const echo_attn_desc_t *desc, const float *dContext, const float *P,
                                  const float *tanh_map, const void *V, const void *v, const int32_t *key_len,
                                  float *dQp, float *dKp, float *dV, float *dv, void *workspace,
                                  size_t workspace_bytes, void *stream) {
    return bwd_impl(desc, dContext, P, tanh_map, true, false, nullptr, nullptr, V, v, key_len, dQp, dKp, dV, dv,
                    workspace, workspace_bytes, stream);
}

void echo_attn_profile_enable(int on) {
    g_prof_on = on != 0;
    if (!on) {
        for (auto &r : g_prof) {
            (void)hipEventDestroy(r.t0);
            (void)hipEventDestroy(r.t1);
        }
        g_prof.clear();
    }
}

int echo_attn_profile_read(const char **names, int *launches, float *total_ms, int cap) {
    int n = 0;
    for (auto &r : g_prof) {
        float ms = 0.f;
        if (hipEventSynchronize(r.t1) == hipSuccess) (void)hipEventElapsedTime(&ms, r.t0, r.t1);
        (void)hipEventDestroy(r.t0);
        (void)hipEventDestroy(r.t1);
        int k = 0;
        for (; k < n && k < cap; ++k)
            if (names[k] == r.name) break;
        if (k == n) {
            if (n < cap) {
                names[n] = r.name;
                launches[n] = 0;
                total_ms[n] = 0.f;
            }
            ++n;
        }
        if (k < cap) {
            launches[k] += 1;
            total_ms[k] += ms;
        }
    }
    g_prof.clear();
    return n;
}

const char *echo_status_string(echo_status_t s) {
    switch (s) {
        case ECHO_OK: return "ok";
        case ECHO_ERR_NULL: return "null pointer";
        case ECHO_ERR_SHAPE: return "bad shape";
        case ECHO_ERR_DTYPE: return "bad dtype";
        case ECHO_ERR_WORKSPACE: return "workspace too small";
        case ECHO_ERR_ALIGN: return "pointer not 16-byte aligned";
        case ECHO_ERR_HIP: return "HIP launch error";
    }
    return "unknown status";
}

const char *echo_last_error_detail(void) { return g_last_error.c_str(); }

const char *echo_version(void) { return "libechoattn 0.1 (gfx950)"; }

}  // extern "C"
