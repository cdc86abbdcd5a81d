// C ABI of the eqat library: argument checking on the host, workspace carving, kernel dispatch.
#include <hip/hip_runtime.h>

#include "../../include/eqat.h"
#include "kernels.h"
#include "prof.h"

#include <atomic>
#include <mutex>
#include <vector>

using eqat::Problem;
using eqat::ProfScope;

namespace eqat {
std::atomic<bool> g_prof_on{false};
namespace {
struct ProfRec { hipEvent_t a, b; int kernel; bool closed; };
std::mutex g_prof_mutex;         // guards the two below
std::vector<ProfRec> g_recs;     // event pairs, reused between profiling sessions
size_t g_used = 0;
}  // namespace
int prof_begin(int kernel, hipStream_t st)
{
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (!g_prof_on.load(std::memory_order_relaxed)) return -1;
    if (g_used == g_recs.size()) {
        ProfRec r{};
        if (hipEventCreate(&r.a) != hipSuccess) { g_prof_on = false; return -1; }
        if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); g_prof_on = false; return -1; }
        g_recs.push_back(r);
    }
    const int rec = (int)g_used++;
    g_recs[rec].kernel = kernel;
    g_recs[rec].closed = false;
    (void)hipEventRecord(g_recs[rec].a, st);
    return rec;
}
void prof_end(int rec, hipStream_t st)
{
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (rec < 0 || (size_t)rec >= g_used) return;             // the session was stopped in between
    (void)hipEventRecord(g_recs[rec].b, st);
    g_recs[rec].closed = true;
}
}  // namespace eqat

namespace {

constexpr int64_t kMaxTensorBytes = (int64_t)1 << 31;   // buffer descriptors and 32-bit offsets

inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }
inline bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline int64_t dsize(int32_t dt) { return dt == EQAT_BF16 ? 2 : 4; }

// Checks everything that does not involve a pointer and fills `p`.  `with_tokens` = the call uses T.
eqat_status check_desc(const eqat_desc *d, bool with_tokens, Problem *p)
{
    if (d == nullptr) return EQAT_ERR_NULL;
    if ((d->act_dtype != EQAT_F32 && d->act_dtype != EQAT_BF16) || (d->w_dtype != EQAT_F32 && d->w_dtype != EQAT_BF16))
        return EQAT_ERR_DTYPE;
    if (d->bits < 2 || d->bits > 4) return EQAT_ERR_BITS;
    const int64_t T = with_tokens ? d->tokens : 0, I = d->in_features, O = d->out_features;
    if (T < 0 || I < 1 || O < 1 || I % 32 != 0) return EQAT_ERR_SHAPE;
    if (I >= kMaxTensorBytes || O >= kMaxTensorBytes || T >= kMaxTensorBytes) return EQAT_ERR_SHAPE;
    if (O * I * dsize(d->w_dtype) >= kMaxTensorBytes) return EQAT_ERR_SHAPE;
    if (with_tokens) {
        if (d->act_dtype == EQAT_BF16 && O % 8 != 0) return EQAT_ERR_SHAPE;
        // the MFMA kernels keep running 32-bit byte offsets that step a few K tiles past the end of a tensor
        if (d->act_dtype == EQAT_BF16 && (I >= ((int64_t)1 << 22) || O >= ((int64_t)1 << 22))) return EQAT_ERR_SHAPE;
        if (T * I * dsize(d->act_dtype) >= kMaxTensorBytes || T * O * dsize(d->act_dtype) >= kMaxTensorBytes)
            return EQAT_ERR_SHAPE;
    }
    int64_t g = d->group;
    if (g == -1) g = I;
    if (g <= 0 || g % 32 != 0 || I % g != 0) return EQAT_ERR_GROUP;
    if (p != nullptr) {
        p->T = T; p->I = I; p->O = O; p->g = g; p->G = I / g; p->bits = d->bits;
        p->act_bf16 = d->act_dtype == EQAT_BF16; p->w_bf16 = d->w_dtype == EQAT_BF16;
    }
    return EQAT_OK;
}

struct WsLayout { size_t codes, clamp, sz, part, dwhat, sk_ctr, sk_ctr_bytes, sk_part, sk_part_bytes, total; };

inline bool op_is_bwd(int op) { return op == EQAT_OP_FQ_BWD || op == EQAT_OP_Q_BWD || op == EQAT_OP_QP_BWD; }
inline bool op_is_prepared(int op) { return op == EQAT_OP_QP_FWD || op == EQAT_OP_QP_BWD; }

// Prepared E2E-QP layer (eqat_qlinear_prepare): codes as the kernels read them, the packed zero points as floats, and
// the arrival counters of the GEMM launches that cut tiles along K (zero, and left zero by every launch).
struct PreparedLayout { size_t codes, zb, sk_ctr, sk_ctr_bytes, total; };

PreparedLayout prepared_layout(const Problem &p)
{
    PreparedLayout l{};
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off += align256(bytes); return at; };
    // bf16 activations: working layout; fp32 activations: the dense stream as it is (that path reads it directly)
    l.codes = take(p.act_bf16 ? eqat::work_code_bytes(p) : (size_t)p.O * p.I * p.bits / 8);
    l.zb = take((size_t)p.O * p.G * 4);
    size_t unused = 0;
    eqat::sk_scratch_bytes(p, true, &unused, &l.sk_ctr_bytes);
    l.sk_ctr = take(l.sk_ctr_bytes);
    l.total = off;
    return l;
}

WsLayout ws_layout(const Problem &p, int op)
{
    WsLayout l{};
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off += align256(bytes); return at; };
    const size_t codes_b = eqat::work_code_bytes(p), clamp_b = (size_t)p.O * p.I / 8, sz_b = (size_t)p.O * p.G * 8;
    const size_t part_b = (size_t)p.O * (p.I / 32) * 4, dwhat_b = (size_t)p.O * p.I * 4;
    const bool bwd = op_is_bwd(op), fq = (op == EQAT_OP_FQ_FWD || op == EQAT_OP_FQ_BWD), prepared = op_is_prepared(op);
    if (p.act_bf16) {
        if (!prepared) l.codes = take(codes_b);       // codes in the working layout (from W, or repacked from the dense stream)
        if (fq && bwd) l.clamp = take(clamp_b);
        l.sz = take(sz_b);                            // (step size, zero point of Eq.(2)) of every group, as the GEMMs read them
        if (bwd && eqat::dw_needs_partials(p)) l.part = take(2 * part_b);
        // GEMM launches that cut tiles along K: arrival counters (cleared by the first kernel of every call; their
        // size and place do not depend on the token count; a prepared layer carries its own) and, last, the
        // accumulator parts (large, sparsely touched, never initialised; present only for shapes whose tiles are cut).
        eqat::sk_scratch_bytes(p, bwd, &l.sk_part_bytes, &l.sk_ctr_bytes);
        if (prepared) l.sk_ctr_bytes = 0;
        l.sk_ctr = take(l.sk_ctr_bytes);
        l.sk_part = take(l.sk_part_bytes);
    } else {
        if (!fq) l.sz = take(sz_b);
        if (bwd) l.dwhat = take(dwhat_b);
    }
    l.total = off;
    return l;
}

eqat_status check_ws(const WsLayout &l, const void *ws, size_t ws_bytes)
{
    if (l.total == 0) return EQAT_OK;
    if (ws == nullptr || ws_bytes < l.total) return EQAT_ERR_WORKSPACE;
    if (!aligned(ws, 256)) return EQAT_ERR_ALIGN;
    return EQAT_OK;
}

inline eqat::SkScratch sk_of(const WsLayout &l, char *w8)
{
    if (l.sk_ctr_bytes == 0) return eqat::SkScratch{nullptr, nullptr};
    return eqat::SkScratch{l.sk_part_bytes != 0 ? reinterpret_cast<float *>(w8 + l.sk_part) : nullptr,
                           reinterpret_cast<uint32_t *>(w8 + l.sk_ctr)};
}


inline eqat_status launch_status() { return hipGetLastError() == hipSuccess ? EQAT_OK : EQAT_ERR_DEVICE; }

#define EQAT_REQUIRE(ptr) do { if ((ptr) == nullptr) return EQAT_ERR_NULL; } while (0)
#define EQAT_ALIGNED(ptr) do { if (!aligned((ptr), 16)) return EQAT_ERR_ALIGN; } while (0)

}  // namespace

extern "C" {

const char *eqat_status_string(int status)
{
    switch (status) {
    case EQAT_OK: return "ok";
    case EQAT_ERR_NULL: return "a required pointer is NULL";
    case EQAT_ERR_SHAPE: return "bad shape (T<0, I or O < 1, I % 32 != 0, with bf16 activations O % 8 != 0 or I or O >= 2^22, or a tensor of 2 GiB or more)";
    case EQAT_ERR_BITS: return "bits must be 2, 3 or 4";
    case EQAT_ERR_GROUP: return "group must be -1 or a positive multiple of 32 that divides in_features";
    case EQAT_ERR_DTYPE: return "unknown dtype";
    case EQAT_ERR_ALIGN: return "pointer not 16-byte aligned (workspace: 256-byte)";
    case EQAT_ERR_WORKSPACE: return "workspace missing or too small";
    case EQAT_ERR_DEVICE: return "HIP launch failed";
    case EQAT_ERR_HYPER: return "optimizer constants out of range (0 <= beta < 1, eps >= 0, step >= 1)";
    default: return "unknown status";
    }
}

eqat_status eqat_validate_desc(const eqat_desc *d) { return check_desc(d, true, nullptr); }

int eqat_profile_kernels(void) { return eqat::PK_COUNT; }

const char *eqat_profile_kernel_name(int k)
{
    static const char *names[] = {"init_minmax", "quantize", "e2e_prepare", "gemm_fwd", "gemm_dx",
                                                "gemm_dw", "reduce_partials", "f32_path", "gemv", "recon_loss", "adamw_update"};
    static_assert(sizeof(names) / sizeof(names[0]) == eqat::PK_COUNT, "one name per kernel class");
    return (k >= 0 && k < eqat::PK_COUNT) ? names[k] : "?";
}

eqat_status eqat_profile_start(void)
{
    std::lock_guard<std::mutex> lock(eqat::g_prof_mutex);
    eqat::g_used = 0;
    eqat::g_prof_on = true;
    return EQAT_OK;
}

eqat_status eqat_profile_stop(double *total_ms, int64_t *launches, int n)
{
    std::lock_guard<std::mutex> lock(eqat::g_prof_mutex);
    eqat::g_prof_on = false;
    const size_t used = eqat::g_used;
    eqat::g_used = 0;
    if (total_ms == nullptr || launches == nullptr) return EQAT_ERR_NULL;
    for (int k = 0; k < n; ++k) { total_ms[k] = 0.0; launches[k] = 0; }
    eqat_status rc = EQAT_OK;
    for (size_t i = 0; i < used; ++i) {
        const eqat::ProfRec &r = eqat::g_recs[i];
        if (!r.closed) continue;                                  // a launch of another thread still under way
        float ms = 0.0f;
        if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) { rc = EQAT_ERR_DEVICE; continue; }
        if (r.kernel >= 0 && r.kernel < n) { total_ms[r.kernel] += ms; launches[r.kernel] += 1; }
    }
    return rc;
}

size_t eqat_packed_w_bytes(const eqat_desc *d)
{
    Problem p;
    if (check_desc(d, false, &p) != EQAT_OK) return 0;
    return (size_t)p.O * p.I * p.bits / 8;
}

size_t eqat_packed_z_bytes(const eqat_desc *d)
{
    Problem p;
    if (check_desc(d, false, &p) != EQAT_OK) return 0;
    return (size_t)p.O * 4 * ((p.G * p.bits + 31) / 32);
}

size_t eqat_workspace_bytes(const eqat_desc *d, int op)
{
    Problem p;
    if (op < EQAT_OP_FQ_FWD || op > EQAT_OP_QP_BWD || check_desc(d, true, &p) != EQAT_OK) return 0;
    return ws_layout(p, op).total;
}

eqat_status eqat_init_minmax(const eqat_desc *d, const void *W, float *s, float *z, void *stream)
{
    Problem p;
    if (eqat_status e = check_desc(d, false, &p)) return e;
    EQAT_REQUIRE(W); EQAT_REQUIRE(s); EQAT_REQUIRE(z);
    EQAT_ALIGNED(W); EQAT_ALIGNED(s); EQAT_ALIGNED(z);
    { ProfScope ps(eqat::PK_INIT_MINMAX, (hipStream_t)stream); eqat::launch_init_minmax(p, W, s, z, (hipStream_t)stream); }
    return launch_status();
}

eqat_status eqat_pack(const eqat_desc *d, const void *W, const float *s, const float *z, uint8_t *Wpacked,
                      uint8_t *zpacked, void *stream)
{
    Problem p;
    if (eqat_status e = check_desc(d, false, &p)) return e;
    EQAT_REQUIRE(W); EQAT_REQUIRE(s); EQAT_REQUIRE(z); EQAT_REQUIRE(Wpacked); EQAT_REQUIRE(zpacked);
    EQAT_ALIGNED(W); EQAT_ALIGNED(s); EQAT_ALIGNED(z); EQAT_ALIGNED(Wpacked); EQAT_ALIGNED(zpacked);
    hipStream_t st = (hipStream_t)stream;
    { ProfScope ps(eqat::PK_QUANTIZE, st); eqat::launch_quantize(p, W, s, z, Wpacked, nullptr, nullptr, zpacked, true, nullptr, 0, st); }
    return launch_status();
}

eqat_status eqat_unpack(const eqat_desc *d, const uint8_t *Wpacked, const uint8_t *zpacked, int32_t *codes,
                        int32_t *zcodes, void *stream)
{
    Problem p;
    if (eqat_status e = check_desc(d, false, &p)) return e;
    if (codes != nullptr) { EQAT_REQUIRE(Wpacked); EQAT_ALIGNED(Wpacked); EQAT_ALIGNED(codes); }
    if (zcodes != nullptr) { EQAT_REQUIRE(zpacked); EQAT_ALIGNED(zpacked); EQAT_ALIGNED(zcodes); }
    eqat::launch_unpack(p, Wpacked, zpacked, codes, zcodes, (hipStream_t)stream);
    return launch_status();
}

}  // extern "C"

// keep: the workspace has the layout of the backward pass and is left holding what Eq.(1) produced (codes, clamp
// bit-plane, (s, zbar) pairs), so that a backward call on the same (W, s, z) need not run Eq.(1) again.
static eqat_status fq_fwd_any(const eqat_desc *d, const void *X, const void *W, const float *s, const float *z, void *Y,
                              void *ws, size_t ws_bytes, void *stream, bool keep, bool kept = false)
{
    Problem p;
    if (eqat_status e = check_desc(d, true, &p)) return e;
    EQAT_REQUIRE(W); EQAT_REQUIRE(s); EQAT_REQUIRE(z);
    if (p.T > 0) { EQAT_REQUIRE(X); EQAT_REQUIRE(Y); }
    EQAT_ALIGNED(X); EQAT_ALIGNED(W); EQAT_ALIGNED(s); EQAT_ALIGNED(z); EQAT_ALIGNED(Y);
    const WsLayout l = ws_layout(p, keep ? EQAT_OP_FQ_BWD : EQAT_OP_FQ_FWD);
    if (eqat_status e = check_ws(l, ws, ws_bytes)) return e;
    if (p.T == 0 && !(keep && p.act_bf16)) return EQAT_OK;
    hipStream_t st = (hipStream_t)stream;
    char *w8 = (char *)ws;
    if (p.act_bf16) {
        const eqat::SkScratch sk = sk_of(l, w8);
        if (!kept) { ProfScope ps(eqat::PK_QUANTIZE, st); eqat::launch_quantize(p, W, s, z, w8 + l.codes, keep ? w8 + l.clamp : nullptr, w8 + l.sz, nullptr, false, sk.counters, (uint32_t)(l.sk_ctr_bytes / 4), st); }
        if (p.T > 0) { ProfScope ps(eqat::PK_GEMM_FWD, st); eqat::launch_mfma_fwd(p, X, w8 + l.codes, w8 + l.sz, Y, sk, st); }
    } else {
        { ProfScope ps(eqat::PK_F32, st); eqat::launch_f32_fwd(p, false, X, W, s, z, Y, st); }
    }
    return launch_status();
}

// kept: the workspace still holds what fq_fwd_any(keep) left there for the same (W, s, z).
static eqat_status fq_bwd_any(const eqat_desc *d, const void *X, const void *W, const float *s, const float *z,
                              const void *dY, void *dX, void *dW, float *ds, float *dz, void *ws, size_t ws_bytes,
                              void *stream, bool kept);

extern "C" {

eqat_status eqat_fq_linear_fwd(const eqat_desc *d, const void *X, const void *W, const float *s, const float *z,
                               void *Y, void *ws, size_t ws_bytes, void *stream)
{
    return fq_fwd_any(d, X, W, s, z, Y, ws, ws_bytes, stream, false);
}

eqat_status eqat_fq_linear_fwd_keep(const eqat_desc *d, const void *X, const void *W, const float *s, const float *z,
                                    void *Y, void *ws, size_t ws_bytes, void *stream)
{
    return fq_fwd_any(d, X, W, s, z, Y, ws, ws_bytes, stream, true);
}

eqat_status eqat_fq_linear_fwd_kept(const eqat_desc *d, const void *X, const void *W, const float *s, const float *z,
                                    void *Y, void *ws, size_t ws_bytes, void *stream)
{
    return fq_fwd_any(d, X, W, s, z, Y, ws, ws_bytes, stream, true, true);
}

eqat_status eqat_fq_linear_bwd(const eqat_desc *d, const void *X, const void *W, const float *s, const float *z,
                               const void *dY, void *dX, void *dW, float *ds, float *dz, void *ws, size_t ws_bytes,
                               void *stream)
{
    return fq_bwd_any(d, X, W, s, z, dY, dX, dW, ds, dz, ws, ws_bytes, stream, false);
}

eqat_status eqat_fq_linear_bwd_kept(const eqat_desc *d, const void *X, const void *W, const float *s, const float *z,
                                    const void *dY, void *dX, void *dW, float *ds, float *dz, void *ws, size_t ws_bytes,
                                    void *stream)
{
    return fq_bwd_any(d, X, W, s, z, dY, dX, dW, ds, dz, ws, ws_bytes, stream, true);
}

}  // extern "C"

static eqat_status fq_bwd_any(const eqat_desc *d, const void *X, const void *W, const float *s, const float *z,
                              const void *dY, void *dX, void *dW, float *ds, float *dz, void *ws, size_t ws_bytes,
                              void *stream, bool kept)
{
    Problem p;
    if (eqat_status e = check_desc(d, true, &p)) return e;
    EQAT_REQUIRE(W); EQAT_REQUIRE(s); EQAT_REQUIRE(z);
    const bool want_w = (dW != nullptr || ds != nullptr || dz != nullptr);
    if (p.T > 0) { EQAT_REQUIRE(dY); if (want_w) EQAT_REQUIRE(X); }
    EQAT_ALIGNED(X); EQAT_ALIGNED(W); EQAT_ALIGNED(s); EQAT_ALIGNED(z); EQAT_ALIGNED(dY);
    EQAT_ALIGNED(dX); EQAT_ALIGNED(dW); EQAT_ALIGNED(ds); EQAT_ALIGNED(dz);
    const WsLayout l = ws_layout(p, EQAT_OP_FQ_BWD);
    if (eqat_status e = check_ws(l, ws, ws_bytes)) return e;
    if (dX == nullptr && !want_w) return EQAT_OK;
    hipStream_t st = (hipStream_t)stream;
    char *w8 = (char *)ws;
    if (p.act_bf16) {
        const eqat::SkScratch sk = sk_of(l, w8);
        if (!kept) { ProfScope ps(eqat::PK_QUANTIZE, st); eqat::launch_quantize(p, W, s, z, w8 + l.codes, w8 + l.clamp, w8 + l.sz, nullptr, false, sk.counters, (uint32_t)(l.sk_ctr_bytes / 4), st); }
        if (dX != nullptr) { ProfScope ps(eqat::PK_GEMM_DX, st); eqat::launch_mfma_dx(p, dY, w8 + l.codes, w8 + l.sz, dX, sk, st); }
        if (want_w)
            eqat::launch_mfma_dw(p, true, X, dY, W, w8 + l.codes, w8 + l.clamp, w8 + l.sz, s, dW, ds, dz,
                                 (float *)(w8 + l.part), sk, st);
    } else {
        ProfScope ps(eqat::PK_F32, st);
        if (dX != nullptr && p.T > 0) eqat::launch_f32_dx(p, false, dY, W, s, z, dX, st);
        if (want_w) eqat::launch_f32_dw(p, true, X, dY, W, s, z, (float *)(w8 + l.dwhat), dW, ds, dz, st);
    }
    return launch_status();
}

// What the E2E-QP GEMMs read: codes (working layout; fp32 activations: the dense stream), the (s, z) pairs, the
// scratch of launches that cut tiles, the array of per-32-column partials of dW, the fp32 dWhat of the fp32 path.
struct QOperands { const void *codes; const void *sz; eqat::SkScratch sk; float *part; float *dwhat; };

static eqat_status qlinear_fwd_run(const Problem &p, const void *X, const float *s, const QOperands &q, void *Y, hipStream_t st)
{
    if (p.T == 0) return launch_status();
    if (p.act_bf16) { ProfScope ps(eqat::PK_GEMM_FWD, st); eqat::launch_mfma_fwd(p, X, q.codes, q.sz, Y, q.sk, st); }
    else { ProfScope ps(eqat::PK_F32, st); eqat::launch_f32_fwd(p, true, X, q.codes, s, q.sz, Y, st); }
    return launch_status();
}

static eqat_status qlinear_bwd_run(const Problem &p, const void *X, const float *s, const QOperands &q, const void *dY,
                                   void *dX, float *ds, float *dz, hipStream_t st)
{
    const bool want_g = (ds != nullptr || dz != nullptr);
    if (p.act_bf16) {
        if (dX != nullptr) { ProfScope ps(eqat::PK_GEMM_DX, st); eqat::launch_mfma_dx(p, dY, q.codes, q.sz, dX, q.sk, st); }
        if (want_g) eqat::launch_mfma_dw(p, false, X, dY, nullptr, q.codes, nullptr, q.sz, s, nullptr, ds, dz, q.part, q.sk, st);
    } else {
        ProfScope ps(eqat::PK_F32, st);
        if (dX != nullptr && p.T > 0) eqat::launch_f32_dx(p, true, dY, q.codes, s, q.sz, dX, st);
        if (want_g) eqat::launch_f32_dw(p, false, X, dY, q.codes, s, q.sz, q.dwhat, nullptr, ds, dz, st);
    }
    return launch_status();
}

// The launch that every E2E-QP call starts with: the (s, z) pairs of the groups (s changes from step to step), z from
// the packed zero points or from floats; with `Wpacked` also the codes into the working layout (bf16 activations; a
// prepared layer has them already); arrival counters cleared (`counters` NULL: a prepared layer's stay at zero).
static void qlinear_prepare_into(const Problem &p, const uint8_t *Wpacked, const float *s, const uint8_t *zpacked,
                                 const float *zfloat, void *codes, void *sz, uint32_t *counters, size_t counter_bytes,
                                 hipStream_t st)
{
    ProfScope ps(eqat::PK_PREPARE, st);
    eqat::launch_e2e_prepare(p, p.act_bf16 ? Wpacked : nullptr, codes, s, zpacked, zfloat, sz, nullptr, counters,
                             (uint32_t)(counter_bytes / 4), st);
}

extern "C" {

// E2E-QP forward / backward; the zero points come packed at N bits (zpacked) or as floats (zfloat), one of the two.
static eqat_status qlinear_fwd_any(const eqat_desc *d, const void *X, const uint8_t *Wpacked, const float *s,
                                   const uint8_t *zpacked, const float *zfloat, void *Y, void *ws, size_t ws_bytes,
                                   void *stream, bool keep = false)
{
    Problem p;
    if (eqat_status e = check_desc(d, true, &p)) return e;
    const void *zany = zpacked != nullptr ? (const void *)zpacked : (const void *)zfloat;   // NULL if the caller's was
    EQAT_REQUIRE(Wpacked); EQAT_REQUIRE(s); EQAT_REQUIRE(zany);
    if (p.T > 0) { EQAT_REQUIRE(X); EQAT_REQUIRE(Y); }
    EQAT_ALIGNED(X); EQAT_ALIGNED(Wpacked); EQAT_ALIGNED(s); EQAT_ALIGNED(zany); EQAT_ALIGNED(Y);
    // keep: backward-sized workspace, left holding the codes in the working layout and the zero points as floats
    const WsLayout l = ws_layout(p, keep ? EQAT_OP_Q_BWD : EQAT_OP_Q_FWD);
    if (eqat_status e = check_ws(l, ws, ws_bytes)) return e;
    if (p.T == 0 && !keep) return EQAT_OK;
    hipStream_t st = (hipStream_t)stream;
    char *w8 = (char *)ws;
    if (!keep && eqat::gemv_applies(p)) { // a few tokens: one HBM-bound kernel on the caller's own packed arrays
        ProfScope ps(eqat::PK_GEMV, st);
        eqat::launch_gemv(p, X, Wpacked, s, zpacked, zfloat, Y, st);
        return launch_status();
    }
    const eqat::SkScratch sk = sk_of(l, w8);
    qlinear_prepare_into(p, Wpacked, s, zpacked, zfloat, w8 + l.codes, w8 + l.sz, sk.counters, l.sk_ctr_bytes, st);
    const QOperands q{p.act_bf16 ? (const void *)(w8 + l.codes) : (const void *)Wpacked, w8 + l.sz, sk, nullptr, nullptr};
    return qlinear_fwd_run(p, X, s, q, Y, st);
}

static eqat_status qlinear_bwd_any(const eqat_desc *d, const void *X, const uint8_t *Wpacked, const float *s,
                                   const uint8_t *zpacked, const float *zfloat, const void *dY, void *dX, float *ds,
                                   float *dz, void *ws, size_t ws_bytes, void *stream, bool kept = false)
{
    Problem p;
    if (eqat_status e = check_desc(d, true, &p)) return e;
    const void *zany = zpacked != nullptr ? (const void *)zpacked : (const void *)zfloat;
    EQAT_REQUIRE(Wpacked); EQAT_REQUIRE(s); EQAT_REQUIRE(zany);
    const bool want_g = (ds != nullptr || dz != nullptr);
    if (p.T > 0) { EQAT_REQUIRE(dY); if (want_g) EQAT_REQUIRE(X); }
    EQAT_ALIGNED(X); EQAT_ALIGNED(Wpacked); EQAT_ALIGNED(s); EQAT_ALIGNED(zany); EQAT_ALIGNED(dY);
    EQAT_ALIGNED(dX); EQAT_ALIGNED(ds); EQAT_ALIGNED(dz);
    const WsLayout l = ws_layout(p, EQAT_OP_Q_BWD);
    if (eqat_status e = check_ws(l, ws, ws_bytes)) return e;
    if (dX == nullptr && !want_g) return EQAT_OK;
    hipStream_t st = (hipStream_t)stream;
    char *w8 = (char *)ws;
    const eqat::SkScratch sk = sk_of(l, w8);
    if (!kept) qlinear_prepare_into(p, Wpacked, s, zpacked, zfloat, w8 + l.codes, w8 + l.sz, sk.counters, l.sk_ctr_bytes, st);
    const QOperands q{p.act_bf16 ? (const void *)(w8 + l.codes) : (const void *)Wpacked, w8 + l.sz, sk,
                      (float *)(w8 + l.part), (float *)(w8 + l.dwhat)};
    return qlinear_bwd_run(p, X, s, q, dY, dX, ds, dz, st);
}

size_t eqat_prepared_bytes(const eqat_desc *d)
{
    Problem p;
    if (check_desc(d, false, &p) != EQAT_OK) return 0;
    p.act_bf16 = d->act_dtype == EQAT_BF16;
    return prepared_layout(p).total;
}

eqat_status eqat_qlinear_prepare(const eqat_desc *d, const uint8_t *Wpacked, const uint8_t *zpacked, void *prepared,
                                 size_t prepared_bytes, void *stream)
{
    Problem p;
    if (eqat_status e = check_desc(d, false, &p)) return e;
    EQAT_REQUIRE(Wpacked); EQAT_REQUIRE(zpacked); EQAT_REQUIRE(prepared);
    EQAT_ALIGNED(Wpacked); EQAT_ALIGNED(zpacked);
    const PreparedLayout l = prepared_layout(p);
    if (prepared_bytes < l.total) return EQAT_ERR_WORKSPACE;
    if (!aligned(prepared, 256)) return EQAT_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    char *p8 = (char *)prepared;
    if (!p.act_bf16 &&
        hipMemcpyAsync(p8 + l.codes, Wpacked, (size_t)p.O * p.I * p.bits / 8, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return EQAT_ERR_DEVICE;
    // codes into the working layout, zero points into floats, counters to zero: one launch
    { ProfScope ps(eqat::PK_PREPARE, st);
      eqat::launch_e2e_prepare(p, p.act_bf16 ? Wpacked : nullptr, p8 + l.codes, nullptr, zpacked, nullptr, nullptr,
                               (float *)(p8 + l.zb), (uint32_t *)(p8 + l.sk_ctr), (uint32_t)(l.sk_ctr_bytes / 4), st); }
    return launch_status();
}

// Operands of a call on a prepared layer; enqueues the small launch that pairs the current step sizes with the zero
// points (`z` NULL: those the layer was prepared with; else trained zero points, as floats) unless the workspace still
// holds the pairs of a forward call that kept them.
static eqat_status prepared_operands(const Problem &p, const void *prepared, const float *s, const float *z, int op, void *ws,
                                     size_t ws_bytes, hipStream_t st, QOperands *q, bool make_pairs = true)
{
    EQAT_REQUIRE(prepared);
    if (!aligned(prepared, 256)) return EQAT_ERR_ALIGN;
    const WsLayout l = ws_layout(p, op);
    if (eqat_status e = check_ws(l, ws, ws_bytes)) return e;
    const PreparedLayout pl = prepared_layout(p);
    char *p8 = (char *)const_cast<void *>(prepared), *w8 = (char *)ws;
    q->codes = p8 + pl.codes;
    q->sz = w8 + l.sz;
    q->sk = eqat::SkScratch{l.sk_part_bytes != 0 ? (float *)(w8 + l.sk_part) : nullptr,
                            pl.sk_ctr_bytes != 0 ? (uint32_t *)(p8 + pl.sk_ctr) : nullptr};
    q->part = (float *)(w8 + l.part);
    q->dwhat = (float *)(w8 + l.dwhat);
    if (make_pairs)
        qlinear_prepare_into(p, nullptr, s, nullptr, z != nullptr ? z : (const float *)(p8 + pl.zb), nullptr, w8 + l.sz, nullptr, 0, st);
    return EQAT_OK;
}

// keep: the workspace has the backward's size and layout, so that a backward call finds the pairs where it looks for them
static eqat_status fwd_prepared_any(const eqat_desc *d, const void *X, const void *prepared, const float *s, const float *z,
                                    void *Y, void *ws, size_t ws_bytes, void *stream, bool keep)
{
    Problem p;
    if (eqat_status e = check_desc(d, true, &p)) return e;
    EQAT_REQUIRE(s);
    if (p.T > 0) { EQAT_REQUIRE(X); EQAT_REQUIRE(Y); }
    EQAT_ALIGNED(X); EQAT_ALIGNED(s); EQAT_ALIGNED(z); EQAT_ALIGNED(Y);
    if (p.T == 0 && !keep) return prepared == nullptr ? EQAT_ERR_NULL : EQAT_OK;
    QOperands q{};
    if (eqat_status e = prepared_operands(p, prepared, s, z, keep ? EQAT_OP_QP_BWD : EQAT_OP_QP_FWD, ws, ws_bytes, (hipStream_t)stream, &q)) return e;
    return qlinear_fwd_run(p, X, s, q, Y, (hipStream_t)stream);
}

eqat_status eqat_qlinear_fwd_prepared(const eqat_desc *d, const void *X, const void *prepared, const float *s, const float *z,
                                      void *Y, void *ws, size_t ws_bytes, void *stream)
{
    return fwd_prepared_any(d, X, prepared, s, z, Y, ws, ws_bytes, stream, false);
}

eqat_status eqat_qlinear_fwd_prepared_keep(const eqat_desc *d, const void *X, const void *prepared, const float *s, const float *z,
                                           void *Y, void *ws, size_t ws_bytes, void *stream)
{
    return fwd_prepared_any(d, X, prepared, s, z, Y, ws, ws_bytes, stream, true);
}

static eqat_status bwd_prepared_any(const eqat_desc *d, const void *X, const void *prepared, const float *s, const float *z,
                                    const void *dY, void *dX, float *ds, float *dz, void *ws, size_t ws_bytes, void *stream,
                                    bool kept)
{
    Problem p;
    if (eqat_status e = check_desc(d, true, &p)) return e;
    EQAT_REQUIRE(s);
    const bool want_g = (ds != nullptr || dz != nullptr);
    if (p.T > 0) { EQAT_REQUIRE(dY); if (want_g) EQAT_REQUIRE(X); }
    EQAT_ALIGNED(X); EQAT_ALIGNED(s); EQAT_ALIGNED(z); EQAT_ALIGNED(dY); EQAT_ALIGNED(dX); EQAT_ALIGNED(ds); EQAT_ALIGNED(dz);
    if (dX == nullptr && !want_g) return prepared == nullptr ? EQAT_ERR_NULL : EQAT_OK;
    QOperands q{};
    if (eqat_status e = prepared_operands(p, prepared, s, z, EQAT_OP_QP_BWD, ws, ws_bytes, (hipStream_t)stream, &q, !kept)) return e;
    return qlinear_bwd_run(p, X, s, q, dY, dX, ds, dz, (hipStream_t)stream);
}

eqat_status eqat_qlinear_bwd_prepared(const eqat_desc *d, const void *X, const void *prepared, const float *s, const float *z,
                                      const void *dY, void *dX, float *ds, float *dz, void *ws, size_t ws_bytes, void *stream)
{
    return bwd_prepared_any(d, X, prepared, s, z, dY, dX, ds, dz, ws, ws_bytes, stream, false);
}

eqat_status eqat_qlinear_bwd_prepared_kept(const eqat_desc *d, const void *X, const void *prepared, const float *s, const float *z,
                                           const void *dY, void *dX, float *ds, float *dz, void *ws, size_t ws_bytes, void *stream)
{
    return bwd_prepared_any(d, X, prepared, s, z, dY, dX, ds, dz, ws, ws_bytes, stream, true);
}

// Test aid (host only): how a fwd / dX / dW launch divides its work.
eqat_status eqat_plan_item(const eqat_desc *d, int gemm, int block, int j, int32_t *item, int32_t *exists)
{
    Problem p;
    if (eqat_status e = check_desc(d, true, &p)) return e;
    if (item == nullptr || exists == nullptr) return EQAT_ERR_NULL;
    if (d->act_dtype != EQAT_BF16) return EQAT_ERR_DTYPE;            // the fp32 path has one workgroup per tile
    const int rc = eqat::plan_item_for_test(p, gemm, block, j, item);
    if (rc < 0) return EQAT_ERR_SHAPE;
    *exists = rc;
    return EQAT_OK;
}

// Test aid: what a forward call that keeps its state, or eqat_qlinear_prepare, left behind, in plain arrays.
eqat_status eqat_unpack_state(const eqat_desc *d, int kind, const void *state, int32_t *codes, uint8_t *clamped, float *zbar,
                              void *stream)
{
    Problem p;
    if (eqat_status e = check_desc(d, false, &p)) return e;
    if (d->act_dtype != EQAT_BF16) return EQAT_ERR_DTYPE;          // the fp32 path keeps no state of this kind
    if (kind < EQAT_STATE_FQ_KEPT || kind > EQAT_STATE_PREPARED) return EQAT_ERR_SHAPE;
    EQAT_REQUIRE(state);
    if (clamped != nullptr && kind != EQAT_STATE_FQ_KEPT) return EQAT_ERR_NULL;    // only Block-AP has a clamp plane
    const char *s8 = (const char *)state;
    hipStream_t st = (hipStream_t)stream;
    if (kind == EQAT_STATE_PREPARED) {
        const PreparedLayout l = prepared_layout(p);
        if (codes != nullptr) eqat::launch_unpack_work(p, s8 + l.codes, nullptr, nullptr, codes, nullptr, nullptr, st);
        if (zbar != nullptr &&
            hipMemcpyAsync(zbar, s8 + l.zb, (size_t)p.O * p.G * 4, hipMemcpyDeviceToDevice, st) != hipSuccess) return EQAT_ERR_DEVICE;
    } else {
        p.T = 1;      // the place of these arrays does not depend on the token count
        const WsLayout l = ws_layout(p, kind == EQAT_STATE_FQ_KEPT ? EQAT_OP_FQ_BWD : EQAT_OP_Q_BWD);
        if (codes != nullptr || clamped != nullptr || zbar != nullptr)
            eqat::launch_unpack_work(p, s8 + l.codes, s8 + l.clamp, s8 + l.sz, codes, clamped, zbar, st);
    }
    return launch_status();
}

eqat_status eqat_qlinear_fwd(const eqat_desc *d, const void *X, const uint8_t *Wpacked, const float *s,
                             const uint8_t *zpacked, void *Y, void *ws, size_t ws_bytes, void *stream)
{
    return qlinear_fwd_any(d, X, Wpacked, s, zpacked, nullptr, Y, ws, ws_bytes, stream);
}

eqat_status eqat_qlinear_bwd(const eqat_desc *d, const void *X, const uint8_t *Wpacked, const float *s,
                             const uint8_t *zpacked, const void *dY, void *dX, float *ds, void *ws, size_t ws_bytes,
                             void *stream)
{
    return qlinear_bwd_any(d, X, Wpacked, s, zpacked, nullptr, dY, dX, ds, nullptr, ws, ws_bytes, stream);
}

eqat_status eqat_qlinear_fwd_keep(const eqat_desc *d, const void *X, const uint8_t *Wpacked, const float *s,
                                  const uint8_t *zpacked, void *Y, void *ws, size_t ws_bytes, void *stream)
{
    return qlinear_fwd_any(d, X, Wpacked, s, zpacked, nullptr, Y, ws, ws_bytes, stream, true);
}

eqat_status eqat_qlinear_bwd_kept(const eqat_desc *d, const void *X, const uint8_t *Wpacked, const float *s,
                                  const uint8_t *zpacked, const void *dY, void *dX, float *ds, void *ws, size_t ws_bytes,
                                  void *stream)
{
    return qlinear_bwd_any(d, X, Wpacked, s, zpacked, nullptr, dY, dX, ds, nullptr, ws, ws_bytes, stream, true);
}

eqat_status eqat_qlinear_fwd_z(const eqat_desc *d, const void *X, const uint8_t *Wpacked, const float *s,
                               const float *z, void *Y, void *ws, size_t ws_bytes, void *stream)
{
    return qlinear_fwd_any(d, X, Wpacked, s, nullptr, z, Y, ws, ws_bytes, stream);
}

eqat_status eqat_qlinear_bwd_z(const eqat_desc *d, const void *X, const uint8_t *Wpacked, const float *s,
                               const float *z, const void *dY, void *dX, float *ds, float *dz, void *ws,
                               size_t ws_bytes, void *stream)
{
    return qlinear_bwd_any(d, X, Wpacked, s, nullptr, z, dY, dX, ds, dz, ws, ws_bytes, stream);
}

// ---- several matrices in one launch --------------------------------------------------------------------------------
// All descriptors of a batch must agree in bits and weight dtype (they select the kernel); everything else may differ.
static eqat_status check_batch(int n, const eqat_desc *descs, Problem *ps)
{
    if (descs == nullptr) return EQAT_ERR_NULL;
    if (n < 1 || n > EQAT_MAX_BATCH) return EQAT_ERR_SHAPE;
    for (int i = 0; i < n; ++i) {
        if (eqat_status e = check_desc(&descs[i], false, &ps[i])) return e;
        if (descs[i].bits != descs[0].bits) return EQAT_ERR_BITS;
        if (descs[i].w_dtype != descs[0].w_dtype || descs[i].act_dtype != descs[0].act_dtype) return EQAT_ERR_DTYPE;
    }
    return EQAT_OK;
}

eqat_status eqat_init_minmax_batched(int n, const eqat_desc *descs, const void *const *W, float *const *s, float *const *z,
                                     void *stream)
{
    Problem ps[EQAT_MAX_BATCH];
    if (eqat_status e = check_batch(n, descs, ps)) return e;
    if (W == nullptr || s == nullptr || z == nullptr) return EQAT_ERR_NULL;
    eqat::InitJob jobs[EQAT_MAX_BATCH];
    for (int i = 0; i < n; ++i) {
        EQAT_REQUIRE(W[i]); EQAT_REQUIRE(s[i]); EQAT_REQUIRE(z[i]);
        EQAT_ALIGNED(W[i]); EQAT_ALIGNED(s[i]); EQAT_ALIGNED(z[i]);
        jobs[i] = eqat::InitJob{ps[i], W[i], s[i], z[i]};
    }
    { ProfScope pr(eqat::PK_INIT_MINMAX, (hipStream_t)stream); eqat::launch_init_minmax_batch(jobs, n, (hipStream_t)stream); }
    return launch_status();
}

eqat_status eqat_pack_batched(int n, const eqat_desc *descs, const void *const *W, const float *const *s,
                              const float *const *z, uint8_t *const *Wpacked, uint8_t *const *zpacked, void *stream)
{
    Problem ps[EQAT_MAX_BATCH];
    if (eqat_status e = check_batch(n, descs, ps)) return e;
    if (W == nullptr || s == nullptr || z == nullptr || Wpacked == nullptr || zpacked == nullptr) return EQAT_ERR_NULL;
    eqat::QuantizeJob jobs[EQAT_MAX_BATCH];
    for (int i = 0; i < n; ++i) {
        EQAT_REQUIRE(W[i]); EQAT_REQUIRE(s[i]); EQAT_REQUIRE(z[i]); EQAT_REQUIRE(Wpacked[i]); EQAT_REQUIRE(zpacked[i]);
        EQAT_ALIGNED(W[i]); EQAT_ALIGNED(s[i]); EQAT_ALIGNED(z[i]); EQAT_ALIGNED(Wpacked[i]); EQAT_ALIGNED(zpacked[i]);
        jobs[i] = eqat::QuantizeJob{ps[i], W[i], s[i], z[i], Wpacked[i], nullptr, nullptr, zpacked[i], nullptr, 0};
    }
    { ProfScope pr(eqat::PK_QUANTIZE, (hipStream_t)stream); eqat::launch_quantize_batch(jobs, n, true, (hipStream_t)stream); }
    return launch_status();
}

eqat_status eqat_fq_quantize_batched(int n, const eqat_desc *descs, const void *const *W, const float *const *s,
                                     const float *const *z, void *const *ws, const size_t *ws_bytes, void *stream)
{
    Problem ps[EQAT_MAX_BATCH];
    if (eqat_status e = check_batch(n, descs, ps)) return e;
    if (W == nullptr || s == nullptr || z == nullptr || ws == nullptr || ws_bytes == nullptr) return EQAT_ERR_NULL;
    eqat::QuantizeJob jobs[EQAT_MAX_BATCH];
    for (int i = 0; i < n; ++i) {
        Problem p;                                        // with the tokens, which the workspace layout may depend on
        if (eqat_status e = check_desc(&descs[i], true, &p)) return e;
        EQAT_REQUIRE(W[i]); EQAT_REQUIRE(s[i]); EQAT_REQUIRE(z[i]);
        EQAT_ALIGNED(W[i]); EQAT_ALIGNED(s[i]); EQAT_ALIGNED(z[i]);
        const WsLayout l = ws_layout(p, EQAT_OP_FQ_BWD);
        if (eqat_status e = check_ws(l, ws[i], ws_bytes[i])) return e;
        char *w8 = (char *)ws[i];
        const eqat::SkScratch sk = sk_of(l, w8);
        jobs[i] = eqat::QuantizeJob{p, W[i], s[i], z[i], w8 + l.codes, w8 + l.clamp, w8 + l.sz, nullptr, sk.counters,
                                    (uint32_t)(l.sk_ctr_bytes / 4)};
    }
    if (!ps[0].act_bf16) return EQAT_OK;                  // the fp32 path keeps nothing
    { ProfScope pr(eqat::PK_QUANTIZE, (hipStream_t)stream); eqat::launch_quantize_batch(jobs, n, false, (hipStream_t)stream); }
    return launch_status();
}

size_t eqat_recon_loss_workspace_bytes(void) { return eqat::recon_loss_ws_bytes(); }

eqat_status eqat_recon_loss(int64_t n, int32_t dtype, const void *Y, const void *Yref, float *loss, void *dY, void *ws,
                            size_t ws_bytes, void *stream)
{
    if (dtype != EQAT_F32 && dtype != EQAT_BF16) return EQAT_ERR_DTYPE;
    if (n < 1) return EQAT_ERR_SHAPE;
    EQAT_REQUIRE(Y); EQAT_REQUIRE(Yref); EQAT_REQUIRE(loss);
    EQAT_ALIGNED(Y); EQAT_ALIGNED(Yref); EQAT_ALIGNED(dY);
    if (!aligned(loss, 4)) return EQAT_ERR_ALIGN;
    if (ws == nullptr || ws_bytes < eqat::recon_loss_ws_bytes()) return EQAT_ERR_WORKSPACE;
    if (!aligned(ws, 256)) return EQAT_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    { ProfScope ps(eqat::PK_LOSS, st); eqat::launch_recon_loss(n, dtype == EQAT_BF16, Y, Yref, loss, dY, static_cast<float *>(ws), st); }
    return launch_status();
}

// ---- eqat_recon_loss for callers that cannot allocate ---------------------------------------------------------------
// The workgroup partials of the loss live in this file-scope device array instead of a caller's workspace.  Every GPU
// the library runs on holds its own copy at its own address; host code never uses the array's name as a pointer, only
// the address hipGetSymbolAddress() returns for the device that is current, looked up once per device and kept.
static __device__ __align__(256) float scratch[2048];
static std::atomic<float *> g_scratch_of_device[64];

static eqat_status scratch_of_current_device(float **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return EQAT_ERR_DEVICE;
    float *p = g_scratch_of_device[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        void *sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || sym == nullptr) {
            (void)hipGetLastError();
            return EQAT_ERR_DEVICE;
        }
        p = static_cast<float *>(sym);
        g_scratch_of_device[dev].store(p, std::memory_order_release);     // every thread finds the same address
    }
    *out = p;
    return EQAT_OK;
}

eqat_status eqat_recon_loss_static(int64_t n, int32_t dtype, const void *Y, const void *Yref, float *loss, void *dY,
                                   void *stream)
{
    if (dtype != EQAT_F32 && dtype != EQAT_BF16) return EQAT_ERR_DTYPE;
    if (n < 1) return EQAT_ERR_SHAPE;
    EQAT_REQUIRE(Y); EQAT_REQUIRE(Yref); EQAT_REQUIRE(loss);
    EQAT_ALIGNED(Y); EQAT_ALIGNED(Yref); EQAT_ALIGNED(dY);
    if (!aligned(loss, 4)) return EQAT_ERR_ALIGN;
    // the launch never uses more partials than eqat_recon_loss_workspace_bytes() holds, whatever n is
    if (eqat::recon_loss_ws_bytes() > sizeof(float) * 2048) return EQAT_ERR_WORKSPACE;
    float *partial = nullptr;
    if (eqat_status e = scratch_of_current_device(&partial)) return e;
    hipStream_t st = (hipStream_t)stream;
    // every partial the second kernel reads is written by the first one of the same call: nothing to clear
    { ProfScope ps(eqat::PK_LOSS, st); eqat::launch_recon_loss(n, dtype == EQAT_BF16, Y, Yref, loss, dY, partial, st); }
    return launch_status();
}

eqat_status eqat_block_ap_update(const eqat_desc *d, const eqat_adamw *h, void *W, float *s, float *z, const void *dW,
                                 const float *ds, const float *dz, float *mW, float *vW, float *ms, float *vs, float *mz,
                                 float *vz, void *stream)
{
    Problem p;
    if (eqat_status e = check_desc(d, false, &p)) return e;
    if (h == nullptr) return EQAT_ERR_NULL;
    if (!(h->beta1 >= 0.f && h->beta1 < 1.f && h->beta2 >= 0.f && h->beta2 < 1.f && h->eps >= 0.f) || h->step < 1)
        return EQAT_ERR_HYPER;
    if (W != nullptr) { EQAT_REQUIRE(dW); EQAT_REQUIRE(mW); EQAT_REQUIRE(vW); EQAT_ALIGNED(W); EQAT_ALIGNED(dW); EQAT_ALIGNED(mW); EQAT_ALIGNED(vW); }
    if (s != nullptr) { EQAT_REQUIRE(ds); EQAT_REQUIRE(ms); EQAT_REQUIRE(vs); EQAT_ALIGNED(s); EQAT_ALIGNED(ds); EQAT_ALIGNED(ms); EQAT_ALIGNED(vs); }
    if (z != nullptr) { EQAT_REQUIRE(dz); EQAT_REQUIRE(mz); EQAT_REQUIRE(vz); EQAT_ALIGNED(z); EQAT_ALIGNED(dz); EQAT_ALIGNED(mz); EQAT_ALIGNED(vz); }
    if (W == nullptr && s == nullptr && z == nullptr) return EQAT_OK;
    const eqat::AdamGroup groups[3] = {
        {W, dW, mW, vW, p.O * p.I, h->lr_w, h->weight_decay_w, p.w_bf16, -__builtin_inff()},
        {s, ds, ms, vs, p.O * p.G, h->lr_q, h->weight_decay_q, false, 1e-10f},      // s > 0 is what Eq.(1) needs
        {z, dz, mz, vz, p.O * p.G, h->lr_q, h->weight_decay_q, false, -__builtin_inff()},
    };
    hipStream_t st = (hipStream_t)stream;
    { ProfScope ps(eqat::PK_UPDATE, st); eqat::launch_adamw(groups, h->beta1, h->beta2, h->eps, h->step, st); }
    return launch_status();
}

}  // extern "C"
