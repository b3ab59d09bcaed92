// C ABI of the MDN library: argument validation, workspace carving, kernel sequencing.
// Declarations and the contract of every entry point are in include/mdn.h.
#include "../../include/mdn.h"
#include "mdn_kernels.h"

#include <hip/hip_runtime.h>
#include <string.h>
#include <vector>

using namespace mdn;

namespace {

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

int check_shape(const mdn_shape *s, bool chunked, Dims *d) {
    if (!s) return MDN_ERR_NULL;
    if (s->dtype != MDN_DTYPE_BF16 && s->dtype != MDN_DTYPE_F32) return MDN_ERR_DTYPE;
    if (s->B < 1 || s->T < 1 || s->H < 1) return MDN_ERR_SHAPE;
    if (!((s->dk == 64 && s->dv == 64) || (s->dk == 128 && s->dv == 128))) return MDN_ERR_SHAPE;
    if (chunked && (s->C != 64 || s->T % 64 != 0)) return MDN_ERR_SHAPE;
    if ((long long)s->B * s->H > (1 << 24) || (long long)s->B * s->T * s->H > (1LL << 31) - 1) return MDN_ERR_SHAPE;
    d->B = s->B; d->T = s->T; d->H = s->H; d->N = s->T / 64; d->BH = s->B * s->H;
    d->dk = s->dk; d->dv = s->dv; d->dtype = s->dtype; d->scale = s->scale;
    return MDN_OK;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Carves consecutive 256-byte aligned regions out of the workspace.
struct Carver {
    char *base;
    size_t off = 0;
    explicit Carver(void *b) : base(static_cast<char *>(b)) {}
    void *take(size_t bytes) {
        void *p = base ? base + off : nullptr;
        off += align_up(bytes);
        return p;
    }
};

struct FwdWs { float *coef; void *KT, *U, *nY, *Z, *Bm; size_t total; };

FwdWs carve_fwd(const Dims &d, void *ws) {
    const size_t es = d.dtype == MDN_DTYPE_F32 ? 4 : 2, nb = (size_t)d.BH * d.N;
    Carver c(ws);
    FwdWs w;
    w.coef = static_cast<float *>(c.take(nb * (size_t)(6 * 64 * sizeof(float))));
    w.KT = c.take(nb * d.dk * 64 * es);
    w.U = c.take(nb * 64 * d.dv * es);
    w.nY = c.take(nb * 64 * d.dk * es);
    w.Z = c.take(nb * 64 * d.dk * es);
    w.Bm = c.take(nb * 4096 * es);
    w.total = c.off;
    return w;
}

// Operands of the reverse pass (what intra mode 1 / 2 writes); lives in the backward workspace or in
// the buffer a training forward keeps for the backward.
struct RevOps { float *coef; void *KT, *QT, *nYT, *ZT, *BmT, *TmT; size_t total; };

RevOps carve_rev(const Dims &d, void *p) {
    const size_t es = d.dtype == MDN_DTYPE_F32 ? 4 : 2, nb = (size_t)d.BH * d.N;
    Carver c(p);
    RevOps w;
    w.coef = static_cast<float *>(c.take(nb * (size_t)(6 * 64 * sizeof(float))));
    w.KT = c.take(nb * d.dk * 64 * es);
    w.QT = c.take(nb * d.dk * 64 * es);
    w.nYT = c.take(nb * d.dk * 64 * es);
    w.ZT = c.take(nb * d.dk * 64 * es);
    w.BmT = c.take(nb * 4096 * es);
    w.TmT = c.take(nb * 4096 * es);
    w.total = c.off;
    return w;
}

struct BwdWs { RevOps ops; void *dstates, *states; size_t total; };

BwdWs carve_bwd(const Dims &d, void *ws) {
    const size_t es = d.dtype == MDN_DTYPE_F32 ? 4 : 2, nb = (size_t)d.BH * d.N;
    BwdWs w;
    w.ops = carve_rev(d, ws);
    Carver c(ws);
    c.off = w.ops.total;
    w.dstates = c.take(nb * 2 * d.dk * d.dv * es);
    w.states = c.take(nb * 2 * d.dk * d.dv * es);
    w.total = c.off;
    return w;
}

int launch_status(hipError_t e) { return e == hipSuccess ? MDN_OK : MDN_ERR_LAUNCH; }

// ---- optional per-kernel timing: event pairs around every launch while enabled
struct TimedLaunch { int id; hipEvent_t start, stop; };
bool g_profiling = false;
std::vector<TimedLaunch> g_timed;

template <typename F> int timed(int id, hipStream_t s, F &&launch) {
    if (!g_profiling) return launch_status(launch());
    TimedLaunch t{id, nullptr, nullptr};
    if (hipEventCreate(&t.start) != hipSuccess || hipEventCreate(&t.stop) != hipSuccess) return MDN_ERR_LAUNCH;
    hipEventRecord(t.start, s);
    const int rc = launch_status(launch());
    hipEventRecord(t.stop, s);
    g_timed.push_back(t);
    return rc;
}

} // namespace

extern "C" {

int mdn_version(void) { return 100; }

int mdn_profile_begin(void) {
    g_profiling = true;
    return MDN_OK;
}

int mdn_profile_end(float *ms, int *launches, int n) {
    g_profiling = false;
    int rc = MDN_OK;
    for (const TimedLaunch &t : g_timed) {
        float e = 0.f;
        if (hipEventSynchronize(t.stop) != hipSuccess || hipEventElapsedTime(&e, t.start, t.stop) != hipSuccess)
            rc = MDN_ERR_LAUNCH;
        else if (t.id < n) {
            if (ms) ms[t.id] += e;
            if (launches) launches[t.id] += 1;
        }
        hipEventDestroy(t.start);
        hipEventDestroy(t.stop);
    }
    g_timed.clear();
    return rc;
}

const char *mdn_strerror(int code) {
    switch (code) {
    case MDN_OK: return "ok";
    case MDN_ERR_NULL: return "a required pointer is NULL";
    case MDN_ERR_SHAPE: return "unsupported shape (need dk = dv in {64,128}, C = 64, T % 64 == 0, sizes >= 1)";
    case MDN_ERR_DTYPE: return "unsupported dtype";
    case MDN_ERR_WORKSPACE: return "workspace too small";
    case MDN_ERR_ALIGN: return "pointer not 16-byte aligned";
    case MDN_ERR_LAUNCH: return "kernel launch failed";
    case MDN_ERR_DEVICE: return "current device is not gfx950";
    default: return "unknown error code";
    }
}

int mdn_workspace_bytes(const mdn_shape *shape, int which, size_t *bytes_out) {
    Dims d;
    if (!bytes_out) return MDN_ERR_NULL;
    int rc = check_shape(shape, true, &d);
    if (rc) return rc;
    if (which == MDN_WS_FWD) *bytes_out = carve_fwd(d, nullptr).total;
    else if (which == MDN_WS_BWD) *bytes_out = carve_bwd(d, nullptr).total;
    else return MDN_ERR_SHAPE;
    return MDN_OK;
}

int mdn_saved_states_bytes(const mdn_shape *shape, size_t *bytes_out) {
    Dims d;
    if (!bytes_out) return MDN_ERR_NULL;
    int rc = check_shape(shape, true, &d);
    if (rc) return rc;
    const size_t es = d.dtype == MDN_DTYPE_F32 ? 4 : 2;
    *bytes_out = (size_t)d.BH * d.N * 2 * d.dk * d.dv * es;
    return MDN_OK;
}

int mdn_saved_operands_bytes(const mdn_shape *shape, size_t *bytes_out) {
    Dims d;
    if (!bytes_out) return MDN_ERR_NULL;
    int rc = check_shape(shape, true, &d);
    if (rc) return rc;
    *bytes_out = carve_rev(d, nullptr).total;
    return MDN_OK;
}

int mdn_chunk_fwd(const mdn_shape *shape, const void *q, const void *k, const void *v, const float *beta,
                  const float *alpha, const float *mu, const float *eta, const float *S0, const float *M0,
                  void *o, float *S_final, float *M_final, void *vt_saved, void *states_saved,
                  void *operands_saved, void *workspace, size_t workspace_bytes, void *stream) {
    Dims d;
    int rc = check_shape(shape, true, &d);
    if (rc) return rc;
    if (!q || !k || !v || !beta || !alpha || !mu || !o || !workspace) return MDN_ERR_NULL;
    const void *ptrs[] = {q, k, v, beta, alpha, mu, eta, S0, M0, o, S_final, M_final, vt_saved, states_saved,
                          operands_saved, workspace};
    for (const void *p : ptrs)
        if (p && misaligned(p)) return MDN_ERR_ALIGN;
    FwdWs w = carve_fwd(d, workspace);
    if (workspace_bytes < w.total) return MDN_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);

    IntraArgs ia = {};
    ia.q = q; ia.k = k; ia.v = v; ia.alpha = alpha; ia.beta = beta; ia.mu = mu; ia.eta = eta;
    ia.coef = w.coef; ia.KT = w.KT; ia.U = w.U; ia.nY = w.nY; ia.Z = w.Z; ia.Bm = w.Bm;
    if (operands_saved) {
        // training forward: one precompute pass writes the reverse pass's operands as well
        const RevOps ro = carve_rev(d, operands_saved);
        ia.coef = ro.coef; ia.KT = ro.KT; ia.QT = ro.QT; ia.nYT = ro.nYT; ia.ZT = ro.ZT; ia.BmT = ro.BmT; ia.TmT = ro.TmT;
    }
    rc = timed(MDN_KERNEL_INTRA_FWD, s, [&] { return launch_intra(d, operands_saved ? 2 : 0, ia, s); });
    if (rc) return rc;

    ScanFwdArgs sa = {};
    sa.q = q; sa.coef = ia.coef; sa.KT = ia.KT; sa.U = w.U; sa.nY = w.nY; sa.Z = w.Z; sa.Bm = w.Bm;
    sa.S0 = S0; sa.M0 = M0; sa.o = o; sa.vt_saved = vt_saved; sa.states_saved = states_saved;
    sa.S_final = S_final; sa.M_final = M_final;
    return timed(MDN_KERNEL_SCAN_FWD, s, [&] { return launch_scan_fwd(d, sa, s); });
}

int mdn_chunk_bwd(const mdn_shape *shape, const void *q, const void *k, const void *v, const float *beta,
                  const float *alpha, const float *mu, const float *eta, const float *S0, const float *M0,
                  const void *vt_saved, const void *states_saved, const void *operands_saved, const void *dO,
                  const float *dS_final,
                  const float *dM_final, void *dq, void *dk, void *dv, float *dbeta, float *dalpha,
                  float *dmu, float *deta, float *dS0, float *dM0, void *workspace, size_t workspace_bytes,
                  void *stream) {
    Dims d;
    int rc = check_shape(shape, true, &d);
    if (rc) return rc;
    if (!q || !k || !v || !beta || !alpha || !mu || !vt_saved || !dO || !dq || !dk || !dv || !dbeta || !dalpha ||
        !dmu || !workspace)
        return MDN_ERR_NULL;
    const void *ptrs[] = {q, k, v, beta, alpha, mu, eta, S0, M0, vt_saved, states_saved, operands_saved, dO, dS_final, dM_final,
                          dq, dk, dv, dbeta, dalpha, dmu, deta, dS0, dM0, workspace};
    for (const void *p : ptrs)
        if (p && misaligned(p)) return MDN_ERR_ALIGN;
    BwdWs w = carve_bwd(d, workspace);
    if (workspace_bytes < w.total) return MDN_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);

    // chunk-local operands in the layouts of the reverse pass: kept by the forward, or recomputed
    RevOps ro = w.ops;
    if (operands_saved) {
        ro = carve_rev(d, const_cast<void *>(operands_saved));
    } else {
        IntraArgs ia = {};
        ia.q = q; ia.k = k; ia.v = v; ia.alpha = alpha; ia.beta = beta; ia.mu = mu; ia.eta = eta;
        ia.coef = ro.coef; ia.KT = ro.KT; ia.QT = ro.QT; ia.nYT = ro.nYT; ia.ZT = ro.ZT; ia.BmT = ro.BmT; ia.TmT = ro.TmT;
        rc = timed(MDN_KERNEL_INTRA_BWD, s, [&] { return launch_intra(d, 1, ia, s); });
        if (rc) return rc;
    }

    // chunk-start states: given by the forward, or reconstructed from V~
    const void *states = states_saved;
    if (!states) {
        RebuildArgs ra = {};
        ra.coef = ro.coef; ra.KT = ro.KT; ra.vt_saved = vt_saved; ra.S0 = S0; ra.M0 = M0; ra.states = w.states;
        rc = timed(MDN_KERNEL_REBUILD, s, [&] { return launch_rebuild(d, ra, s); });
        if (rc) return rc;
        states = w.states;
    }

    ScanBwdArgs sb = {};
    sb.k = k; sb.dO = dO; sb.coef = ro.coef; sb.QT = ro.QT; sb.nYT = ro.nYT; sb.ZT = ro.ZT; sb.BmT = ro.BmT;
    sb.TmT = ro.TmT; sb.dS_final = dS_final; sb.dM_final = dM_final; sb.dv = dv; sb.dstates = w.dstates;
    sb.dS0 = dS0; sb.dM0 = dM0;
    rc = timed(MDN_KERNEL_SCAN_BWD, s, [&] { return launch_scan_bwd(d, sb, s); });
    if (rc) return rc;

    GradArgs ga = {};
    ga.q = q; ga.k = k; ga.alpha = alpha; ga.beta = beta; ga.mu = mu; ga.eta = eta;
    ga.vt_saved = vt_saved; ga.dO = dO; ga.dv = dv; ga.KT = ro.KT; ga.QT = ro.QT;
    ga.states = states; ga.dstates = w.dstates;
    ga.dq = dq; ga.dk = dk; ga.dalpha = dalpha; ga.dbeta = dbeta; ga.dmu = dmu; ga.deta = deta;
    return timed(MDN_KERNEL_GRAD, s, [&] { return launch_grad(d, ga, s); });
}

int mdn_recurrent_step(const mdn_shape *shape, const void *q, const void *k, const void *v, const float *beta,
                       const float *alpha, const float *mu, const float *eta, float *S, float *M, void *o,
                       void *stream) {
    Dims d;
    int rc = check_shape(shape, false, &d);
    if (rc) return rc;
    if (!q || !k || !v || !beta || !alpha || !mu || !S || !M || !o) return MDN_ERR_NULL;
    const void *ptrs[] = {q, k, v, beta, alpha, mu, eta, S, M, o};
    for (const void *p : ptrs)
        if (p && misaligned(p)) return MDN_ERR_ALIGN;
    RecurrentArgs ra = {};
    ra.q = q; ra.k = k; ra.v = v; ra.alpha = alpha; ra.beta = beta; ra.mu = mu; ra.eta = eta;
    ra.S = S; ra.M = M; ra.o = o;
    hipStream_t s = static_cast<hipStream_t>(stream);
    return timed(MDN_KERNEL_RECURRENT, s, [&] { return launch_recurrent(d, ra, s); });
}

} // extern "C"
