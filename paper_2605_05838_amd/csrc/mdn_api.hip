// C ABI of the MDN library: argument validation, workspace carving, kernel sequencing.
// Declarations and the contract of every entry point are in include/mdn.h.
#include "../../include/mdn.h"
#include "mdn_kernels.h"

#include <hip/hip_runtime.h>
#include <string.h>
#include <atomic>
#include <mutex>
#include <type_traits>
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
    if (chunked && s->C != 64 && s->C != 32 && s->C != 16) return MDN_ERR_SHAPE;
    // (chunks of 16 or 32 tokens run as 64-token tiles: up to 4 rows per token)
    const long long tile = chunked ? 64 / s->C : 1;
    if ((long long)s->B * s->H > (1 << 24) || ((long long)s->B * s->T + 64) * s->H * tile > (1LL << 31) - 1) return MDN_ERR_SHAPE;
    d->B = s->B; d->T = s->T; d->H = s->H; d->N = s->T / 64; d->BH = s->B * s->H; // N: the FULL chunks
    d->n0 = 0; d->n1 = d->N;
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

struct FwdWs { float *coef; void *KT, *Tm, *Bm; float *carryS, *carryM; size_t total; };

FwdWs carve_fwd(const Dims &d, void *ws) {
    const size_t es = d.dtype == MDN_DTYPE_F32 ? 4 : 2, nb = (size_t)d.BH * d.N;
    Carver c(ws);
    FwdWs w;
    w.coef = static_cast<float *>(c.take(nb * (size_t)(64 * kCoefBlockCols * sizeof(float))));
    w.KT = scan_fwd_reads_KT(d) ? c.take(nb * d.dk * 64 * es) : nullptr; // (16-bit storage: made on chip from the k rows)
    w.Tm = c.take(nb * 4096 * es);
    w.Bm = c.take(nb * 4096 * es);
    // states handed from one segment of the sequence to the next when the call is split (see segments())
    w.carryS = static_cast<float *>(c.take((size_t)d.BH * d.dk * d.dv * sizeof(float)));
    w.carryM = static_cast<float *>(c.take((size_t)d.BH * d.dk * d.dv * sizeof(float)));
    w.total = c.off;
    return w;
}

// Operands of the reverse pass (what intra mode 1 / 2 writes); lives in the backward workspace or in
// the buffer a training forward keeps for the backward.
struct RevOps { float *coef; void *KT, *QT, *BmT, *TmT; size_t total; };

RevOps carve_rev(const Dims &d, void *p) {
    const size_t es = d.dtype == MDN_DTYPE_F32 ? 4 : 2, nb = (size_t)d.BH * d.N;
    Carver c(p);
    RevOps w;
    w.coef = static_cast<float *>(c.take(nb * (size_t)(64 * kCoefBlockCols * sizeof(float))));
    w.KT = c.take(nb * d.dk * 64 * es);
    w.QT = c.take(nb * d.dk * 64 * es);
    w.BmT = c.take(nb * 4096 * es);
    w.TmT = c.take(nb * 4096 * es);
    w.total = c.off;
    return w;
}

struct BwdWs { RevOps ops; void *dstates, *states, *dstates_lo, *states_lo; float *carryS, *carryM; size_t total; };

// `precise`: room for the rounding remainders of the two state tensors as well (16-bit storage, calls that bring
// adjoints of the final states in; see precise_call)
BwdWs carve_bwd(const Dims &d, void *ws, bool precise) {
    const size_t es = d.dtype == MDN_DTYPE_F32 ? 4 : 2, nb = (size_t)d.BH * d.N;
    BwdWs w;
    w.ops = carve_rev(d, ws);
    Carver c(ws);
    c.off = w.ops.total;
    w.dstates = c.take(nb * 2 * d.dk * d.dv * es);
    w.states = c.take(nb * 2 * d.dk * d.dv * es);
    w.dstates_lo = precise ? c.take(nb * 2 * d.dk * d.dv * es) : nullptr;
    w.states_lo = precise ? c.take(nb * 2 * d.dk * d.dv * es) : nullptr;
    w.carryS = static_cast<float *>(c.take((size_t)d.BH * d.dk * d.dv * sizeof(float)));
    w.carryM = static_cast<float *>(c.take((size_t)d.BH * d.dk * d.dv * sizeof(float)));
    w.total = c.off;
    return w;
}

// ---- a sequence length that is not a multiple of 64: the full chunks run on the caller's tensors (d.N counts
// them, d.T stays the row stride between sequences), the partial last chunk on padded copies (see mdn_tail.hip)
Dims tail_dims(const Dims &d) {
    Dims t = d;
    t.T = 64; t.N = 1; t.n0 = 0; t.n1 = 1;
    return t;
}

size_t elem_size(const Dims &d) { return d.dtype == MDN_DTYPE_F32 ? 4 : 2; }
size_t saved_states_part(const Dims &d) { return (size_t)d.BH * d.N * 2 * d.dk * d.dv * elem_size(d); }

// padded [B,64,H,*] copies of the partial chunk's tensors, and the states handed between the two parts
struct TailBufs {
    void *q, *k, *v, *o, *vt, *dO, *dq, *dk, *dv;
    float *beta, *alpha, *mu, *eta, *dbeta, *dalpha, *dmu, *deta;
    float *S_mid, *M_mid, *dS_mid, *dM_mid;
    size_t total;
};

TailBufs carve_tail(const Dims &d, bool backward, void *p) {
    const size_t es = elem_size(d), rows = (size_t)d.B * 64 * d.H, st = (size_t)d.BH * d.dk * d.dv * sizeof(float);
    Carver c(p);
    TailBufs t = {};
    t.q = c.take(rows * d.dk * es);
    t.k = c.take(rows * d.dk * es);
    t.v = c.take(rows * d.dv * es);
    t.vt = c.take(rows * d.dv * es);
    t.beta = static_cast<float *>(c.take(rows * 4));
    t.alpha = static_cast<float *>(c.take(rows * 4));
    t.mu = static_cast<float *>(c.take(rows * 4));
    t.eta = static_cast<float *>(c.take(rows * 4));
    t.S_mid = static_cast<float *>(c.take(st));
    t.M_mid = static_cast<float *>(c.take(st));
    if (!backward) {
        t.o = c.take(rows * d.dv * es);
    } else {
        t.dO = c.take(rows * d.dv * es);
        t.dq = c.take(rows * d.dk * es);
        t.dk = c.take(rows * d.dk * es);
        t.dv = c.take(rows * d.dv * es);
        t.dbeta = static_cast<float *>(c.take(rows * 4));
        t.dalpha = static_cast<float *>(c.take(rows * 4));
        t.dmu = static_cast<float *>(c.take(rows * 4));
        t.deta = static_cast<float *>(c.take(rows * 4));
        t.dS_mid = static_cast<float *>(c.take(st));
        t.dM_mid = static_cast<float *>(c.take(st));
    }
    t.total = c.off;
    return t;
}

void *offset(void *p, size_t bytes) { return p ? static_cast<char *>(p) + bytes : nullptr; }
const void *offset(const void *p, size_t bytes) { return p ? static_cast<const char *>(p) + bytes : nullptr; }

struct TailList {
    TailCopy c;
    TailList(const Dims &d, int r) {
        c = {};
        c.B = d.B; c.T = d.T; c.H = d.H; c.t0 = d.N * 64; c.r = r;
    }
    void add(const void *full, void *padded, size_t row_bytes, float pad = 0.f) {
        if (!full || !padded) return;
        TailTensor &t = c.t[c.n++];
        t.full = full; t.padded = padded; t.row_bytes = (int)row_bytes;
        memcpy(&t.pad_word, &pad, 4); // (0.f and 1.f are also right for the 16-bit rows: only 0 is used there)
    }
};

int launch_status(hipError_t e) { return e == hipSuccess ? MDN_OK : MDN_ERR_LAUNCH; }

// ---- optional per-kernel timing: event pairs around every launch while enabled.  The list of pairs is shared by
// all threads of the process and guarded by a mutex.
struct TimedLaunch { int id; hipEvent_t start, stop; };
std::atomic<bool> g_profiling{false};
std::atomic<int> g_profile_period{1};          // every period-th launch is bracketed
std::atomic<unsigned> g_profile_seen{0};       // launches since mdn_profile_begin
std::atomic<int> g_launched[MDN_KERNEL_COUNT]; // all launches per kernel id since mdn_profile_begin
std::mutex g_timed_mutex;
std::vector<TimedLaunch> g_timed;

// this thread is inside the entry point that must not allocate: no timing events, no second stream
thread_local bool t_no_alloc = false;

template <typename F> int timed(int id, hipStream_t s, F &&launch) {
    if (t_no_alloc || !g_profiling.load(std::memory_order_relaxed)) return launch_status(launch());
    if (id >= 0 && id < MDN_KERNEL_COUNT) g_launched[id].fetch_add(1, std::memory_order_relaxed);
    const unsigned seen = g_profile_seen.fetch_add(1, std::memory_order_relaxed);
    if (seen % (unsigned)g_profile_period.load(std::memory_order_relaxed) != 0) return launch_status(launch());
    TimedLaunch t{id, nullptr, nullptr};
    if (hipEventCreate(&t.start) != hipSuccess || hipEventCreate(&t.stop) != hipSuccess) return MDN_ERR_LAUNCH;
    const bool r0 = hipEventRecord(t.start, s) == hipSuccess;
    const int rc = launch_status(launch());
    const bool r1 = hipEventRecord(t.stop, s) == hipSuccess;
    {
        std::lock_guard<std::mutex> lock(g_timed_mutex);
        g_timed.push_back(t);
    }
    return r0 && r1 ? rc : MDN_ERR_LAUNCH;
}

// ---- splitting a call into segments of the sequence.  When the serial scans occupy at most half of the CUs
// (few (batch, head) pairs, long sequences), the chunk-parallel kernel of segment i+1 (forward) or of segment
// i (backward) runs beside the scan of the neighbouring segment, on a second stream of the library's own:
// the scan's workgroups leave the other CUs to it.  States cross a segment boundary through two small fp32
// buffers in the workspace.
std::atomic<int> g_segments{0}; // 0: automatic
// this thread is inside a pair of calls that run beside each other on the two streams: no segments inside them
thread_local bool t_side_stream_taken = false;

// the serial scans of a call would occupy at most half of the CUs
bool few_scan_workgroups(const Dims &d) { return 2 * scan_workgroups(d) <= num_cus(); }

int segments(const Dims &d) {
    int k;
    if (t_side_stream_taken || t_no_alloc) return 1;
    const int forced = g_segments.load(std::memory_order_relaxed);
    if (forced > 0) {
        k = forced;
    } else {
        k = (few_scan_workgroups(d) && d.N >= 32) ? 4 : 1;
    }
    if (k > d.N / 4) k = d.N / 4;
    return k < 1 ? 1 : (k > 16 ? 16 : k);
}

// The library's second stream and its events, one set per device, shared by every call on that device.  A call that
// uses them holds the device's mutex while it ENQUEUES (the kernels themselves run after it has returned): an event
// is recorded and waited for inside one such section, so calls from several host threads cannot interleave their
// record / wait pairs; their work on the second stream is simply ordered one call after the other.
struct Side {
    hipStream_t stream = nullptr;
    std::vector<hipEvent_t> ev;
    std::recursive_mutex mutex; // (recursive: two calls beside each other take it, then each call inside may again)
};

// the second stream and n events on the current device (created once, default priority); call with the lock held
Side *side_device() {
    static Side per_device[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    return &per_device[dev];
}
Side *side(int n) {
    Side *xp = side_device();
    if (!xp) return nullptr;
    Side &x = *xp;
    if (!x.stream && hipStreamCreateWithFlags(&x.stream, hipStreamNonBlocking) != hipSuccess) return nullptr;
    while ((int)x.ev.size() < n) {
        hipEvent_t e;
        if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return nullptr;
        x.ev.push_back(e);
    }
    return &x;
}

Dims segment(const Dims &d, int i, int k) {
    Dims r = d;
    r.n0 = (int)((long long)d.N * i / k);
    r.n1 = (int)((long long)d.N * (i + 1) / k);
    return r;
}

// ---- the forward over the chunks [0, d.N) of the tensors in `c`
struct FwdCall {
    const void *q, *k, *v;
    const float *beta, *alpha, *mu, *eta, *S0, *M0;
    void *o;
    float *S_final, *M_final;
    void *vt_saved, *states_saved, *operands_saved;
    void *states_lo; // rounding remainders of states_saved (16-bit storage), or null; see packed_final_states
};

int run_fwd(const Dims &d, const FwdCall &c, const FwdWs &w, hipStream_t s) {
    int rc;
    IntraArgs ia = {};
    ia.q = c.q; ia.k = c.k; ia.alpha = c.alpha; ia.beta = c.beta; ia.mu = c.mu; ia.eta = c.eta;
    ia.coef = w.coef; ia.KT = w.KT; ia.Tm = w.Tm; ia.Bm = w.Bm;
    if (c.operands_saved) {
        // training forward: one precompute pass writes the reverse pass's operands as well
        const RevOps ro = carve_rev(d, c.operands_saved);
        ia.coef = ro.coef; ia.KT = ro.KT; ia.QT = ro.QT; ia.BmT = ro.BmT; ia.TmT = ro.TmT;
    }
    ScanFwdArgs sa = {};
    sa.q = c.q; sa.k = c.k; sa.v = c.v; sa.coef = ia.coef; sa.KT = ia.KT; sa.Tm = w.Tm; sa.Bm = w.Bm;
    sa.S0 = c.S0; sa.M0 = c.M0; sa.o = c.o; sa.vt_saved = c.vt_saved; sa.states_saved = c.states_saved;
    sa.states_lo = c.states_lo;
    sa.S_final = c.S_final; sa.M_final = c.M_final;
    // K^T for this forward alone: not written if its scan forms K^T out of the k rows itself
    if (!c.operands_saved && !scan_fwd_reads_KT(d)) ia.KT = nullptr, sa.KT = nullptr;
    const int mode = c.operands_saved ? 2 : 0;
    const int nseg = segments(d);
    if (nseg == 1) {
        rc = timed(MDN_KERNEL_INTRA_FWD, s, [&] { return launch_intra(d, mode, ia, s); });
        if (rc) return rc;
        return timed(MDN_KERNEL_SCAN_FWD, s, [&] { return launch_scan_fwd(d, sa, s); });
    }
    // segments: precompute of segment i+1 on the second stream beside the scan of segment i on the caller's
    Side *sdev = side_device();
    if (!sdev) return MDN_ERR_LAUNCH;
    std::lock_guard<std::recursive_mutex> lock(sdev->mutex);
    Side *sd = side(nseg + 1);
    if (!sd) return MDN_ERR_LAUNCH;
    if (hipEventRecord(sd->ev[nseg], s) != hipSuccess || hipStreamWaitEvent(sd->stream, sd->ev[nseg], 0) != hipSuccess)
        return MDN_ERR_LAUNCH; // whatever the caller's stream holds so far comes first
    // (from here on the second stream holds work of this call: whatever happens, the caller's stream waits for it
    //  before the call returns, so that "complete when the stream reaches the end of the call" also holds for a
    //  call that fails half-way)
    for (int i = 0; i < nseg; ++i) {
        const Dims di = segment(d, i, nseg);
        rc = timed(MDN_KERNEL_INTRA_FWD, sd->stream, [&] { return launch_intra(di, mode, ia, sd->stream); });
        const bool joined = hipEventRecord(sd->ev[i], sd->stream) == hipSuccess && hipStreamWaitEvent(s, sd->ev[i], 0) == hipSuccess;
        if (rc) return rc;
        if (!joined) return MDN_ERR_LAUNCH;
        sa.S0 = i == 0 ? c.S0 : w.carryS;
        sa.M0 = i == 0 ? c.M0 : w.carryM;
        sa.S_final = i == nseg - 1 ? c.S_final : w.carryS;
        sa.M_final = i == nseg - 1 ? c.M_final : w.carryM;
        rc = timed(MDN_KERNEL_SCAN_FWD, s, [&] { return launch_scan_fwd(di, sa, s); });
        if (rc) return rc; // (every launch on the second stream so far has been joined above)
    }
    return MDN_OK;
}

// ---- the backward over the chunks [0, d.N) of the tensors in `c`, in two steps: what does not depend on the
// adjoints coming in from the right (the reverse pass's operands, the chunk-start states), then the rest
struct BwdCall {
    const void *q, *k, *v;
    const float *beta, *alpha, *mu, *eta, *S0, *M0;
    const void *vt_saved, *states_saved, *operands_saved, *dO;
    const float *dS_final, *dM_final;
    void *dq, *dk, *dv;
    float *dbeta, *dalpha, *dmu, *deta, *dS0, *dM0;
};
struct Prepared {
    RevOps ro;
    const void *states;
};

// Adjoints of the final states that come in from outside can be large against everything dO puts into the states;
// the sums of dk dv products that they enter (the state traces, the products with V~) then carry the 16-bit storage
// rounding of the chunk states and chunk adjoints at full weight.  Such a call keeps the rounding remainders of both
// tensors as well (which also means it reconstructs the states rather than taking the forward's 16-bit copy).
bool precise_call(const Dims &d, const BwdCall &c) {
    return d.dtype == MDN_DTYPE_BF16 && (c.dS_final || c.dM_final);
}

// S_after, M_after (or null): the states after the last chunk, which the reconstruction can hand on
int bwd_prepare(const Dims &d, const BwdCall &c, const BwdWs &w, float *S_after, float *M_after, hipStream_t s,
                Prepared *out, bool precise) {
    int rc;
    // chunk-local operands in the layouts of the reverse pass: kept by the forward, or recomputed
    out->ro = w.ops;
    if (c.operands_saved) {
        out->ro = carve_rev(d, const_cast<void *>(c.operands_saved));
    } else {
        IntraArgs ia = {};
        ia.q = c.q; ia.k = c.k; ia.alpha = c.alpha; ia.beta = c.beta; ia.mu = c.mu; ia.eta = c.eta;
        ia.coef = out->ro.coef; ia.KT = out->ro.KT; ia.QT = out->ro.QT; ia.BmT = out->ro.BmT; ia.TmT = out->ro.TmT;
        rc = timed(MDN_KERNEL_INTRA_BWD, s, [&] { return launch_intra(d, 1, ia, s); });
        if (rc) return rc;
    }
    // chunk-start states: given by the forward, or reconstructed from V~
    out->states = precise ? nullptr : c.states_saved;
    if (!out->states) {
        RebuildArgs ra = {};
        ra.coef = out->ro.coef; ra.k = c.k; ra.KT = out->ro.KT; ra.vt_saved = c.vt_saved; ra.S0 = c.S0; ra.M0 = c.M0;
        ra.states = w.states; ra.states_lo = precise ? w.states_lo : nullptr; ra.S_final = S_after; ra.M_final = M_after;
        rc = timed(MDN_KERNEL_REBUILD, s, [&] { return launch_rebuild(d, ra, s); });
        if (rc) return rc;
        out->states = w.states;
    }
    return MDN_OK;
}

int bwd_run(const Dims &d, const BwdCall &c, const BwdWs &w, const Prepared &p, hipStream_t s, bool precise) {
    int rc;
    const RevOps &ro = p.ro;
    ScanBwdArgs sb = {};
    sb.k = c.k; sb.dO = c.dO; sb.coef = ro.coef; sb.QT = ro.QT; sb.KT = ro.KT; sb.BmT = ro.BmT;
    sb.TmT = ro.TmT; sb.dS_final = c.dS_final; sb.dM_final = c.dM_final; sb.dv = c.dv; sb.dstates = w.dstates;
    sb.dS0 = c.dS0; sb.dM0 = c.dM0; sb.dstates_lo = precise ? w.dstates_lo : nullptr;
    GradArgs ga = {};
    ga.q = c.q; ga.k = c.k; ga.alpha = c.alpha; ga.beta = c.beta; ga.mu = c.mu; ga.eta = c.eta;
    ga.vt_saved = c.vt_saved; ga.dO = c.dO; ga.dv = c.dv; ga.KT = ro.KT; ga.QT = ro.QT;
    ga.states = p.states; ga.dstates = w.dstates;
    ga.states_lo = precise ? w.states_lo : nullptr; ga.dstates_lo = precise ? w.dstates_lo : nullptr;
    ga.dq = c.dq; ga.dk = c.dk; ga.dalpha = c.dalpha; ga.dbeta = c.dbeta; ga.dmu = c.dmu; ga.deta = c.deta;
    const int nseg = segments(d);
    if (nseg == 1) {
        rc = timed(MDN_KERNEL_SCAN_BWD, s, [&] { return launch_scan_bwd(d, sb, s); });
        if (rc) return rc;
        return timed(MDN_KERNEL_GRAD, s, [&] { return launch_grad(d, ga, s); });
    }
    // segments, last first: the gradient kernel of segment i on the second stream beside the reverse scan
    // of segment i-1 on the caller's; the caller's stream then waits for the last gradient launch
    Side *sdev = side_device();
    if (!sdev) return MDN_ERR_LAUNCH;
    std::lock_guard<std::recursive_mutex> lock(sdev->mutex);
    Side *sd = side(nseg + 1);
    if (!sd) return MDN_ERR_LAUNCH;
    rc = MDN_OK;
    for (int i = nseg - 1; i >= 0 && !rc; --i) {
        const Dims di = segment(d, i, nseg);
        sb.dS_final = i == nseg - 1 ? c.dS_final : w.carryS;
        sb.dM_final = i == nseg - 1 ? c.dM_final : w.carryM;
        sb.dS0 = i == 0 ? c.dS0 : w.carryS;
        sb.dM0 = i == 0 ? c.dM0 : w.carryM;
        rc = timed(MDN_KERNEL_SCAN_BWD, s, [&] { return launch_scan_bwd(di, sb, s); });
        if (rc) break;
        if (hipEventRecord(sd->ev[i], s) != hipSuccess || hipStreamWaitEvent(sd->stream, sd->ev[i], 0) != hipSuccess) {
            rc = MDN_ERR_LAUNCH;
            break;
        }
        rc = timed(MDN_KERNEL_GRAD, sd->stream, [&] { return launch_grad(di, ga, sd->stream); });
    }
    // the caller's stream waits for whatever went to the second stream, also when a launch failed on the way
    if (hipEventRecord(sd->ev[nseg], sd->stream) != hipSuccess || hipStreamWaitEvent(s, sd->ev[nseg], 0) != hipSuccess)
        return MDN_ERR_LAUNCH;
    return rc;
}

size_t fwd_ws_total(const Dims &d, int r) {
    if (r == 0) return carve_fwd(d, nullptr).total;
    return carve_fwd(d, nullptr).total + carve_fwd(tail_dims(d), nullptr).total + carve_tail(d, false, nullptr).total;
}
size_t bwd_ws_total(const Dims &d, int r, bool precise) {
    if (r == 0) return carve_bwd(d, nullptr, precise).total;
    return carve_bwd(d, nullptr, precise).total + carve_bwd(tail_dims(d), nullptr, precise).total +
           carve_tail(d, true, nullptr).total;
}

// The forward over a sequence of any length: d.N full chunks and r = T % 64 tokens of a partial one.
int fwd_any(const Dims &d, int r, FwdCall c, void *workspace, hipStream_t s) {
    int rc;
    const FwdWs w = carve_fwd(d, workspace);
    if (r == 0) return run_fwd(d, c, w, s);

    // full chunks on the caller's tensors, then the partial chunk on padded copies
    const Dims dt = tail_dims(d);
    const FwdWs wt = carve_fwd(dt, offset(workspace, w.total));
    const TailBufs tb = carve_tail(d, false, offset(workspace, w.total + wt.total));
    const size_t es = elem_size(d);
    float *S_final = c.S_final, *M_final = c.M_final;
    void *o = c.o;
    if (d.N > 0) {
        c.S_final = tb.S_mid;
        c.M_final = tb.M_mid;
        rc = run_fwd(d, c, w, s);
        if (rc) return rc;
    }
    TailList in(d, r);
    in.add(c.q, tb.q, d.dk * es);
    in.add(c.k, tb.k, d.dk * es);
    in.add(c.v, tb.v, d.dv * es);
    in.add(c.beta, tb.beta, 4, 0.f);
    in.add(c.alpha, tb.alpha, 4, 1.f);
    in.add(c.mu, tb.mu, 4, 1.f);
    in.add(c.eta, tb.eta, 4, 1.f);
    rc = launch_status(launch_tail_copy(in.c, true, s));
    if (rc) return rc;
    FwdCall ct = {tb.q, tb.k, tb.v, tb.beta, tb.alpha, tb.mu, c.eta ? tb.eta : nullptr,
                  d.N > 0 ? tb.S_mid : c.S0, d.N > 0 ? tb.M_mid : c.M0, tb.o, S_final, M_final,
                  c.vt_saved ? tb.vt : nullptr, offset(c.states_saved, saved_states_part(d)),
                  offset(c.operands_saved, carve_rev(d, nullptr).total), offset(c.states_lo, saved_states_part(d))};
    rc = run_fwd(dt, ct, wt, s);
    if (rc) return rc;
    TailList out(d, r);
    out.add(o, tb.o, d.dv * es);
    out.add(c.vt_saved, tb.vt, d.dv * es);
    return launch_status(launch_tail_copy(out.c, false, s));
}

// The backward over a sequence of any length (see fwd_any).
int bwd_any(const Dims &d, int r, BwdCall c, void *workspace, hipStream_t s) {
    int rc;
    const BwdCall u = c; // the caller's pointers (c is redirected for the full chunks below)
    const bool precise = precise_call(d, u);
    const BwdWs w = carve_bwd(d, workspace, precise);
    Prepared pm;
    if (r == 0) {
        rc = bwd_prepare(d, c, w, nullptr, nullptr, s, &pm, precise);
        return rc ? rc : bwd_run(d, c, w, pm, s, precise);
    }

    // the partial chunk comes last in the sequence, so first in the reverse pass; what it needs from the full
    // chunks (the states they leave) is ready after their preparation step
    const Dims dt = tail_dims(d);
    const BwdWs wt = carve_bwd(dt, offset(workspace, w.total), precise);
    const TailBufs tb = carve_tail(d, true, offset(workspace, w.total + wt.total));
    const size_t es = elem_size(d);
    if (d.N > 0) {
        rc = bwd_prepare(d, c, w, tb.S_mid, tb.M_mid, s, &pm, precise);
        if (rc) return rc;
    }
    TailList in(d, r);
    in.add(u.q, tb.q, d.dk * es);
    in.add(u.k, tb.k, d.dk * es);
    in.add(u.v, tb.v, d.dv * es);
    in.add(u.vt_saved, tb.vt, d.dv * es);
    in.add(u.dO, tb.dO, d.dv * es);
    in.add(u.beta, tb.beta, 4, 0.f);
    in.add(u.alpha, tb.alpha, 4, 1.f);
    in.add(u.mu, tb.mu, 4, 1.f);
    in.add(u.eta, tb.eta, 4, 1.f);
    rc = launch_status(launch_tail_copy(in.c, true, s));
    if (rc) return rc;
    // (with states kept by the forward the partial chunk's start states are in their own part of that buffer;
    //  otherwise they are reconstructed from what the full chunks leave)
    BwdCall ct = {tb.q, tb.k, tb.v, tb.beta, tb.alpha, tb.mu, u.eta ? tb.eta : nullptr,
                  d.N > 0 ? tb.S_mid : u.S0, d.N > 0 ? tb.M_mid : u.M0, tb.vt,
                  offset(u.states_saved, saved_states_part(d)), offset(u.operands_saved, carve_rev(d, nullptr).total), tb.dO,
                  u.dS_final, u.dM_final, tb.dq, tb.dk, tb.dv, tb.dbeta, tb.dalpha, tb.dmu, u.deta ? tb.deta : nullptr,
                  d.N > 0 ? tb.dS_mid : u.dS0, d.N > 0 ? tb.dM_mid : u.dM0};
    Prepared pt;
    rc = bwd_prepare(dt, ct, wt, nullptr, nullptr, s, &pt, precise);
    if (rc) return rc;
    rc = bwd_run(dt, ct, wt, pt, s, precise);
    if (rc) return rc;
    if (d.N > 0) {
        c.dS_final = tb.dS_mid;
        c.dM_final = tb.dM_mid;
        rc = bwd_run(d, c, w, pm, s, precise);
        if (rc) return rc;
    }
    TailList out(d, r);
    out.add(u.dq, tb.dq, d.dk * es);
    out.add(u.dk, tb.dk, d.dk * es);
    out.add(u.dv, tb.dv, d.dv * es);
    out.add(u.dbeta, tb.dbeta, 4);
    out.add(u.dalpha, tb.dalpha, 4);
    out.add(u.dmu, tb.dmu, 4);
    out.add(u.deta, tb.deta, 4);
    return launch_status(launch_tail_copy(out.c, false, s));
}

// ---- chunk sizes below 64 (Algorithm 1 lists C in {16, 32, 64}).  The kernels are built around 64-token tiles (four
// waves of 16 tokens, 64-lane coefficient scans), so a chunk of C < 64 tokens runs as one such tile whose rows from C on
// are identity steps of the recurrence (k = v = q = 0, alpha = mu = 1, beta = 0, dO = 0: they change no state and pass
// every adjoint through, see the partial last chunk above): the chunk-local coefficients, the triangular solve and the
// state hand-over are exactly those of Algorithm 1 at chunk size C, at 64 / C times the work of the C = 64 path.
// The tokens are expanded into padded copies in the workspace and the results collected from them.
Dims expanded_dims(const Dims &d, int C) {
    Dims e = d;
    const int NC = (d.T + C - 1) / C;
    e.T = NC * 64; e.N = NC; e.n0 = 0; e.n1 = NC;
    return e;
}

struct ExpBufs {
    void *q, *k, *v, *o, *vt, *dO, *dq, *dk, *dv;
    float *beta, *alpha, *mu, *eta, *dbeta, *dalpha, *dmu, *deta;
    void *rest;
    size_t total;
};

ExpBufs carve_exp(const Dims &e, bool backward, bool precise, void *p) {
    const size_t es = elem_size(e), rows = (size_t)e.B * e.T * e.H;
    Carver c(p);
    ExpBufs x = {};
    x.q = c.take(rows * e.dk * es);
    x.k = c.take(rows * e.dk * es);
    x.v = c.take(rows * e.dv * es);
    x.vt = c.take(rows * e.dv * es);
    x.beta = static_cast<float *>(c.take(rows * 4));
    x.alpha = static_cast<float *>(c.take(rows * 4));
    x.mu = static_cast<float *>(c.take(rows * 4));
    x.eta = static_cast<float *>(c.take(rows * 4));
    if (!backward) {
        x.o = c.take(rows * e.dv * es);
        x.rest = c.take(fwd_ws_total(e, 0));
    } else {
        x.dO = c.take(rows * e.dv * es);
        x.dq = c.take(rows * e.dk * es);
        x.dk = c.take(rows * e.dk * es);
        x.dv = c.take(rows * e.dv * es);
        x.dbeta = static_cast<float *>(c.take(rows * 4));
        x.dalpha = static_cast<float *>(c.take(rows * 4));
        x.dmu = static_cast<float *>(c.take(rows * 4));
        x.deta = static_cast<float *>(c.take(rows * 4));
        x.rest = c.take(bwd_ws_total(e, 0, precise));
    }
    x.total = c.off;
    return x;
}

struct ChunkList {
    ChunkCopy c;
    ChunkList(const Dims &d, int C) {
        c = {};
        c.B = d.B; c.T = d.T; c.H = d.H; c.C = C; c.NC = (d.T + C - 1) / C;
    }
    void add(const void *full, void *padded, size_t row_bytes, float pad = 0.f) {
        if (!full || !padded) return;
        TailTensor &t = c.t[c.n++];
        t.full = full; t.padded = padded; t.row_bytes = (int)row_bytes;
        memcpy(&t.pad_word, &pad, 4);
    }
};

int fwd_small_chunks(const Dims &d, int C, const FwdCall &c, void *workspace, hipStream_t s) {
    const Dims e = expanded_dims(d, C);
    const ExpBufs x = carve_exp(e, false, false, workspace);
    const size_t es = elem_size(d);
    ChunkList in(d, C);
    in.add(c.q, x.q, d.dk * es);
    in.add(c.k, x.k, d.dk * es);
    in.add(c.v, x.v, d.dv * es);
    in.add(c.beta, x.beta, 4, 0.f);
    in.add(c.alpha, x.alpha, 4, 1.f);
    in.add(c.mu, x.mu, 4, 1.f);
    in.add(c.eta, x.eta, 4, 1.f);
    int rc = launch_status(launch_chunk_copy(in.c, true, s));
    if (rc) return rc;
    const FwdCall ce = {x.q, x.k, x.v, x.beta, x.alpha, x.mu, c.eta ? x.eta : nullptr, c.S0, c.M0, x.o, c.S_final, c.M_final,
                        c.vt_saved ? x.vt : nullptr, c.states_saved, c.operands_saved};
    rc = run_fwd(e, ce, carve_fwd(e, x.rest), s);
    if (rc) return rc;
    ChunkList out(d, C);
    out.add(c.o, x.o, d.dv * es);
    out.add(c.vt_saved, x.vt, d.dv * es);
    return launch_status(launch_chunk_copy(out.c, false, s));
}

int bwd_small_chunks(const Dims &d, int C, const BwdCall &c, void *workspace, hipStream_t s) {
    const Dims e = expanded_dims(d, C);
    const bool precise = precise_call(d, c);
    const ExpBufs x = carve_exp(e, true, precise, workspace);
    const size_t es = elem_size(d);
    ChunkList in(d, C);
    in.add(c.q, x.q, d.dk * es);
    in.add(c.k, x.k, d.dk * es);
    in.add(c.v, x.v, d.dv * es);
    in.add(c.vt_saved, x.vt, d.dv * es);
    in.add(c.dO, x.dO, d.dv * es);
    in.add(c.beta, x.beta, 4, 0.f);
    in.add(c.alpha, x.alpha, 4, 1.f);
    in.add(c.mu, x.mu, 4, 1.f);
    in.add(c.eta, x.eta, 4, 1.f);
    int rc = launch_status(launch_chunk_copy(in.c, true, s));
    if (rc) return rc;
    const BwdCall ce = {x.q, x.k, x.v, x.beta, x.alpha, x.mu, c.eta ? x.eta : nullptr, c.S0, c.M0, x.vt, c.states_saved,
                        c.operands_saved, x.dO, c.dS_final, c.dM_final, x.dq, x.dk, x.dv, x.dbeta, x.dalpha, x.dmu,
                        c.deta ? x.deta : nullptr, c.dS0, c.dM0};
    const BwdWs w = carve_bwd(e, x.rest, precise);
    Prepared pm;
    rc = bwd_prepare(e, ce, w, nullptr, nullptr, s, &pm, precise);
    if (rc) return rc;
    rc = bwd_run(e, ce, w, pm, s, precise);
    if (rc) return rc;
    ChunkList out(d, C);
    out.add(c.dq, x.dq, d.dk * es);
    out.add(c.dk, x.dk, d.dk * es);
    out.add(c.dv, x.dv, d.dv * es);
    out.add(c.dbeta, x.dbeta, 4);
    out.add(c.dalpha, x.dalpha, 4);
    out.add(c.dmu, x.dmu, 4);
    out.add(c.deta, x.deta, 4);
    return launch_status(launch_chunk_copy(out.c, false, s));
}

// workspace, kept states and kept operands of a call, whatever its chunk size
size_t fwd_ws_call(const Dims &d, const mdn_shape *shape) {
    if (shape->C == 64) return fwd_ws_total(d, shape->T % 64);
    return carve_exp(expanded_dims(d, shape->C), false, false, nullptr).total;
}
size_t bwd_ws_call(const Dims &d, const mdn_shape *shape, bool precise) {
    if (shape->C == 64) return bwd_ws_total(d, shape->T % 64, precise);
    return carve_exp(expanded_dims(d, shape->C), true, precise, nullptr).total;
}

// ---- packed variable-length batches: the sequences lie one after another along T of a [1, T, H, *] tensor;
// sequence i is tokens [cu[i], cu[i+1]).  Each sequence runs as a batch of one through the any-length path
// (stream order makes the shared workspace safe).
int check_varlen(const mdn_shape *shape, const int32_t *cu, int32_t n_seq, Dims *d) {
    const int rc = check_shape(shape, true, d);
    if (rc) return rc;
    if (shape->C != 64) return MDN_ERR_SHAPE; // (packed batches: chunk size 64 only)
    if (!cu) return MDN_ERR_NULL;
    if (shape->B != 1 || n_seq < 1 || cu[0] != 0 || cu[n_seq] != shape->T) return MDN_ERR_SHAPE;
    for (int i = 0; i < n_seq; ++i)
        if (cu[i + 1] <= cu[i]) return MDN_ERR_SHAPE;
    return MDN_OK;
}

Dims seq_dims(const Dims &all, int len) {
    Dims d = all;
    d.B = 1; d.T = len; d.N = len / 64; d.BH = all.H; d.n0 = 0; d.n1 = d.N;
    return d;
}

// ---- the same batch as ONE stream of tokens.  By Eq. Mt.recurrent / St.recurrent a token with alpha = mu = 0
// sees nothing of the states before it (e = v, M = -eta k e^T, S = -beta M: what a sequence that starts from zero
// states computes at its first token, whose own alpha and mu multiply those zeros and do not matter), and passes no
// adjoint back to them.  So with alpha and mu set to zero at the first token of every sequence but the first, the
// whole batch is one sequence of shape->T tokens: one set of launches, however many and however short the sequences,
// and no partial chunk but the last.  Open to calls that neither give nor ask for per-sequence states; the
// gradients of the zeroed gates are zero (they multiply zero states) and are set so.
// When the stream's scans would leave half of the CUs idle (few heads), it is cut in two at the sequence start nearest
// to its middle and the halves run beside each other, one on the caller's stream and one on the library's second
// stream: nothing passes between them, the state is cut there anyway.
struct PackedWs { float *alpha, *mu; void *rest, *rest2; int cut; size_t total; };

// index m (0 < m < n_seq) of the sequence that starts the second half, or 0: no cut
int packed_cut(const Dims &d, const int32_t *cu, int n_seq) {
    if (n_seq < 2 || !few_scan_workgroups(d) || d.T < 2048) return 0;
    int best = 1;
    for (int i = 1; i < n_seq; ++i)
        if (llabs(2LL * cu[i] - d.T) < llabs(2LL * cu[best] - d.T)) best = i;
    // (a lopsided cut would only take the overlap of the chunk-parallel kernels with the scans away from the long half)
    const int small = cu[best] < d.T - cu[best] ? cu[best] : d.T - cu[best];
    return small >= d.T / 4 ? best : 0;
}

PackedWs carve_packed(const Dims &d, const int32_t *cu, int n_seq, bool backward, void *ws) {
    Carver c(ws);
    PackedWs w = {};
    w.alpha = static_cast<float *>(c.take((size_t)d.T * d.H * sizeof(float)));
    w.mu = static_cast<float *>(c.take((size_t)d.T * d.H * sizeof(float)));
    w.cut = packed_cut(d, cu, n_seq);
    auto need = [&](int len) {
        const Dims p = seq_dims(d, len);
        return backward ? bwd_ws_total(p, len % 64, false) : fwd_ws_total(p, len % 64);
    };
    if (w.cut) {
        w.rest = c.take(need(cu[w.cut]));
        w.rest2 = c.take(need(d.T - cu[w.cut]));
    } else {
        w.rest = c.take(need(d.T));
    }
    w.total = c.off;
    return w;
}

// the two halves beside each other: first(stream), second(stream) are the two calls
template <typename F1, typename F2> int run_beside(hipStream_t s, F1 &&first, F2 &&second) {
    constexpr int E0 = 30, E1 = 31; // (the events below these belong to the segments of a single call)
    Side *sdev = side_device();
    if (!sdev) return MDN_ERR_LAUNCH;
    std::lock_guard<std::recursive_mutex> lock(sdev->mutex);
    Side *sd = side(E1 + 1);
    if (!sd) return MDN_ERR_LAUNCH;
    if (hipEventRecord(sd->ev[E0], s) != hipSuccess || hipStreamWaitEvent(sd->stream, sd->ev[E0], 0) != hipSuccess)
        return MDN_ERR_LAUNCH; // whatever the caller's stream holds so far comes first
    t_side_stream_taken = true;
    int rc = first(s);
    if (!rc) rc = second(sd->stream);
    t_side_stream_taken = false;
    if (hipEventRecord(sd->ev[E1], sd->stream) != hipSuccess || hipStreamWaitEvent(s, sd->ev[E1], 0) != hipSuccess)
        return MDN_ERR_LAUNCH;
    return rc;
}

// value at the first tokens of sequences 1 .. n_seq-1 of a (and b)
int set_at_sequence_starts(const Dims &d, const int32_t *cu, int n_seq, float *a, float *b, float value, hipStream_t s) {
    SeqStarts st;
    st.H = d.H;
    for (int i = 1; i < n_seq;) {
        st.n = 0;
        while (i < n_seq && st.n < kSeqStartsPerLaunch) st.t[st.n++] = cu[i++];
        if (launch_set_at_tokens(a, b, value, st, s) != hipSuccess) return MDN_ERR_LAUNCH;
    }
    return MDN_OK;
}

// copies of alpha, mu with the sequence starts zeroed
int packed_gates(const Dims &d, const int32_t *cu, int n_seq, const float *alpha, const float *mu, const PackedWs &w,
                 hipStream_t s) {
    const size_t bytes = (size_t)d.T * d.H * sizeof(float);
    if (hipMemcpyAsync(w.alpha, alpha, bytes, hipMemcpyDeviceToDevice, s) != hipSuccess ||
        hipMemcpyAsync(w.mu, mu, bytes, hipMemcpyDeviceToDevice, s) != hipSuccess)
        return MDN_ERR_LAUNCH;
    return set_at_sequence_starts(d, cu, n_seq, w.alpha, w.mu, 0.f, s);
}

// ---- the stream form with per-sequence FINAL states (zero initial states): the stream keeps its chunk-start
// states; the state after a sequence's last token is that of the chunk holding the token, run once more from its
// start state over the tokens up to the sequence's end, the rest of the chunk padded with tokens that change no state
// (as for a partial last chunk).  All sequences' last chunks form one batch of n_seq rows of 64 tokens.
Dims rows_dims(const Dims &d, int n_seq) {
    Dims t = tail_dims(d);
    t.B = n_seq; t.BH = n_seq * d.H;
    return t;
}

// one half of the stream (or all of it): sequences [seq0, seq1), tokens [t0, t0 + len)
struct StreamPiece {
    int seq0, seq1, t0, len;
    void *states; // its chunk-start states (full chunks, then the partial chunk's block)
    void *states_lo; // 16-bit storage: what the rounding of `states` dropped (the final states start from hi + lo)
    void *rest;   // its forward workspace
};

struct PackedFinalWs {
    PackedWs g;       // gate copies
    int npieces;
    StreamPiece piece[2];
    void *k, *v, *o;  // padded rows [n_seq, 64, H, *]
    float *beta, *alpha, *mu, *eta, *S0, *M0;
    void *rest_rows;
    size_t total;
};

PackedFinalWs carve_packed_final(const Dims &d, const int32_t *cu, int n_seq, void *ws) {
    const size_t es = elem_size(d), rows = (size_t)n_seq * 64 * d.H, st = (size_t)n_seq * d.H * d.dk * d.dv * sizeof(float);
    const Dims dr = rows_dims(d, n_seq);
    Carver c(ws);
    PackedFinalWs w = {};
    w.g.alpha = static_cast<float *>(c.take((size_t)d.T * d.H * sizeof(float)));
    w.g.mu = static_cast<float *>(c.take((size_t)d.T * d.H * sizeof(float)));
    const int cut = packed_cut(d, cu, n_seq);
    w.npieces = cut ? 2 : 1;
    w.piece[0] = {0, cut ? cut : n_seq, 0, cut ? cu[cut] : d.T, nullptr, nullptr, nullptr};
    w.piece[1] = {cut, n_seq, cut ? cu[cut] : 0, cut ? d.T - cu[cut] : 0, nullptr, nullptr, nullptr};
    for (int p = 0; p < w.npieces; ++p) {
        const Dims dp = seq_dims(d, w.piece[p].len);
        const size_t sb = saved_states_part(dp) + (dp.T % 64 ? saved_states_part(tail_dims(dp)) : 0);
        w.piece[p].states = c.take(sb);
        w.piece[p].states_lo = d.dtype == MDN_DTYPE_BF16 ? c.take(sb) : nullptr;
        w.piece[p].rest = c.take(fwd_ws_total(dp, dp.T % 64));
    }
    w.k = c.take(rows * d.dk * es);
    w.v = c.take(rows * d.dv * es);
    w.o = c.take(rows * d.dv * es);
    w.beta = static_cast<float *>(c.take(rows * 4));
    w.alpha = static_cast<float *>(c.take(rows * 4));
    w.mu = static_cast<float *>(c.take(rows * 4));
    w.eta = static_cast<float *>(c.take(rows * 4));
    w.S0 = static_cast<float *>(c.take(st));
    w.M0 = static_cast<float *>(c.take(st));
    w.rest_rows = c.take(fwd_ws_total(dr, 0));
    w.total = c.off;
    return w;
}

int packed_final_states(const Dims &d, const int32_t *cu, int n_seq, const FwdCall &stream, const PackedFinalWs &w,
                        float *S_final, float *M_final, hipStream_t s) {
    const size_t es = elem_size(d), st = (size_t)d.H * d.dk * d.dv;
    for (int p = 0; p < w.npieces; ++p) {
        const StreamPiece &pc = w.piece[p];
        const Dims dp = seq_dims(d, pc.len); // (the piece's chunks count from its own first token)
        for (int i0 = pc.seq0; i0 < pc.seq1; i0 += kSeqRowsPerLaunch) {
            const int n = pc.seq1 - i0 < kSeqRowsPerLaunch ? pc.seq1 - i0 : kSeqRowsPerLaunch;
            const size_t rows0 = (size_t)i0 * 64 * d.H;
            SeqRows g = {};
            SeqChunks sc = {};
            g.n = sc.n = n; g.H = sc.H = d.H;
            sc.N = dp.N; sc.dk = d.dk; sc.dv = d.dv; sc.dtype = d.dtype;
            for (int e = 0; e < n; ++e) {
                const int end = cu[i0 + e + 1] - pc.t0, chunk = (end - 1) / 64;
                sc.chunk[e] = chunk;
                g.t0[e] = pc.t0 + chunk * 64;
                g.r[e] = end - chunk * 64;
            }
            auto add = [&](const void *full, void *padded, size_t row_bytes, float pad) {
                if (!full) return;
                TailTensor &t = g.t[g.ntens++];
                t.full = full; t.padded = static_cast<char *>(padded) + rows0 * row_bytes; t.row_bytes = (int)row_bytes;
                memcpy(&t.pad_word, &pad, 4);
            };
            add(stream.k, w.k, d.dk * es, 0.f);
            add(stream.v, w.v, d.dv * es, 0.f);
            add(stream.beta, w.beta, 4, 0.f);
            add(stream.alpha, w.alpha, 4, 1.f);
            add(stream.mu, w.mu, 4, 1.f);
            add(stream.eta, w.eta, 4, 1.f);
            if (launch_gather_seq_rows(g, s) != hipSuccess) return MDN_ERR_LAUNCH;
            if (launch_states_to_f32(pc.states, offset(pc.states, saved_states_part(dp)), pc.states_lo,
                                     offset(pc.states_lo, saved_states_part(dp)), sc, w.S0 + (size_t)i0 * st,
                                     w.M0 + (size_t)i0 * st, s) != hipSuccess)
                return MDN_ERR_LAUNCH;
        }
    }
    // (the rows' outputs o are of no use: q is given the k rows, o a scratch tensor)
    const Dims dr = rows_dims(d, n_seq);
    FwdCall c = {w.k, w.k, w.v, w.beta, w.alpha, w.mu, stream.eta ? w.eta : nullptr, w.S0, w.M0, w.o, S_final, M_final,
                 nullptr, nullptr, nullptr};
    return run_fwd(dr, c, carve_fwd(dr, w.rest_rows), s);
}

// ---- the forward's workspace as a fixed array in device memory, for callers that cannot allocate.  Every GPU the
// library runs on holds its own copy of the array (at its own address) until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress: the address it returns, per device, is what is passed on.
static __device__ __align__(256) unsigned char scratch[MDN_NOALLOC_SCRATCH_BYTES];

// device address of `scratch` on the current device (asked for once per device, with that device current)
int scratch_address(void **out) {
    static std::mutex mutex;
    static void *per_device[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MDN_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(mutex);
    if (!per_device[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MDN_ERR_DEVICE;
        per_device[dev] = p;
    }
    *out = per_device[dev];
    return MDN_OK;
}

template <typename P> P *at_token(P *base, size_t token, size_t bytes_per_token) {
    return base ? reinterpret_cast<P *>(reinterpret_cast<char *>(const_cast<typename std::remove_const<P>::type *>(base)) +
                                        token * bytes_per_token)
                : nullptr;
}

} // namespace

extern "C" {

int mdn_version(void) { return 200; }

int mdn_set_segments(int k) { return g_segments.exchange(k < 0 ? 0 : k); }

int mdn_profile_begin_sampled(int period) {
    if (period < 1) return MDN_ERR_SHAPE;
    g_profile_period.store(period);
    g_profile_seen.store(0);
    for (auto &c : g_launched) c.store(0);
    g_profiling.store(true);
    return MDN_OK;
}

int mdn_profile_begin(void) { return mdn_profile_begin_sampled(1); }

int mdn_profile_launch_counts(int *launched, int n) {
    if (!launched) return MDN_ERR_NULL;
    for (int i = 0; i < n && i < MDN_KERNEL_COUNT; ++i) launched[i] = g_launched[i].load();
    return MDN_OK;
}

int mdn_profile_end(float *ms, int *launches, int n) {
    g_profiling.store(false);
    int rc = MDN_OK;
    std::vector<TimedLaunch> taken;
    {
        std::lock_guard<std::mutex> lock(g_timed_mutex);
        taken.swap(g_timed);
    }
    for (const TimedLaunch &t : taken) {
        float e = 0.f;
        if (hipEventSynchronize(t.stop) != hipSuccess || hipEventElapsedTime(&e, t.start, t.stop) != hipSuccess)
            rc = MDN_ERR_LAUNCH;
        else if (t.id < n) {
            if (ms) ms[t.id] += e;
            if (launches) launches[t.id] += 1;
        }
        if (hipEventDestroy(t.start) != hipSuccess || hipEventDestroy(t.stop) != hipSuccess) rc = MDN_ERR_LAUNCH;
    }
    return rc;
}

const char *mdn_strerror(int code) {
    switch (code) {
    case MDN_OK: return "ok";
    case MDN_ERR_NULL: return "a required pointer is NULL";
    case MDN_ERR_SHAPE: return "unsupported shape (need dk = dv in {64,128}, C in {16,32,64}, sizes >= 1)";
    case MDN_ERR_DTYPE: return "unsupported dtype";
    case MDN_ERR_WORKSPACE: return "workspace too small (or, for mdn_chunk_fwd_noalloc, the shape needs more than its fixed scratch array)";
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
    if (which == MDN_WS_FWD) *bytes_out = fwd_ws_call(d, shape);
    else if (which == MDN_WS_BWD) *bytes_out = bwd_ws_call(d, shape, false);
    else if (which == MDN_WS_BWD_STATE_ADJOINTS) *bytes_out = bwd_ws_call(d, shape, d.dtype == MDN_DTYPE_BF16);
    else return MDN_ERR_SHAPE;
    return MDN_OK;
}

int mdn_saved_states_bytes(const mdn_shape *shape, size_t *bytes_out) {
    Dims d;
    if (!bytes_out) return MDN_ERR_NULL;
    int rc = check_shape(shape, true, &d);
    if (rc) return rc;
    // the full chunks' blocks first, then (T % 64 != 0) one block per (batch, head) for the partial chunk
    if (shape->C != 64) *bytes_out = saved_states_part(expanded_dims(d, shape->C));
    else *bytes_out = saved_states_part(d) + (shape->T % 64 ? saved_states_part(tail_dims(d)) : 0);
    return MDN_OK;
}

int mdn_saved_operands_bytes(const mdn_shape *shape, size_t *bytes_out) {
    Dims d;
    if (!bytes_out) return MDN_ERR_NULL;
    int rc = check_shape(shape, true, &d);
    if (rc) return rc;
    if (shape->C != 64) *bytes_out = carve_rev(expanded_dims(d, shape->C), nullptr).total;
    else *bytes_out = carve_rev(d, nullptr).total + (shape->T % 64 ? carve_rev(tail_dims(d), nullptr).total : 0);
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
    const int r = shape->T % 64;
    if (workspace_bytes < fwd_ws_call(d, shape)) return MDN_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    FwdCall c = {q, k, v, beta, alpha, mu, eta, S0, M0, o, S_final, M_final, vt_saved, states_saved, operands_saved};
    if (shape->C != 64) return fwd_small_chunks(d, shape->C, c, workspace, s);
    return fwd_any(d, r, c, workspace, s);
}

int mdn_chunk_fwd_noalloc(const mdn_shape *shape, const void *q, const void *k, const void *v, const float *beta,
                          const float *alpha, const float *mu, const float *eta, const float *S0, const float *M0,
                          void *o, float *S_final, float *M_final, void *vt_saved, void *stream) {
    Dims d;
    int rc = check_shape(shape, true, &d);
    if (rc) return rc;
    if (!q || !k || !v || !beta || !alpha || !mu || !o) return MDN_ERR_NULL;
    const void *ptrs[] = {q, k, v, beta, alpha, mu, eta, S0, M0, o, S_final, M_final, vt_saved};
    for (const void *p : ptrs)
        if (p && misaligned(p)) return MDN_ERR_ALIGN;
    const int r = shape->T % 64;
    if (fwd_ws_call(d, shape) > (size_t)MDN_NOALLOC_SCRATCH_BYTES) return MDN_ERR_WORKSPACE;
    void *ws = nullptr;
    rc = scratch_address(&ws);
    if (rc) return rc;
    // Nothing in the forward's workspace has to start from zero: the chunk-local operands are written in full by the
    // chunk-parallel kernel before the scan reads them, the padded copies of a partial chunk by the gather kernel.
    FwdCall c = {q, k, v, beta, alpha, mu, eta, S0, M0, o, S_final, M_final, vt_saved, nullptr, nullptr};
    t_no_alloc = true; // one stream, no timing events: nothing below creates a stream, an event or memory
    rc = shape->C != 64 ? fwd_small_chunks(d, shape->C, c, ws, static_cast<hipStream_t>(stream))
                        : fwd_any(d, r, c, ws, static_cast<hipStream_t>(stream));
    t_no_alloc = false;
    return rc;
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
    const int r = shape->T % 64;
    BwdCall c = {q, k, v, beta, alpha, mu, eta, S0, M0, vt_saved, states_saved, operands_saved, dO, dS_final, dM_final,
                 dq, dk, dv, dbeta, dalpha, dmu, deta, dS0, dM0};
    if (workspace_bytes < bwd_ws_call(d, shape, precise_call(d, c))) return MDN_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (shape->C != 64) return bwd_small_chunks(d, shape->C, c, workspace, s);
    return bwd_any(d, r, c, workspace, s);
}

int mdn_workspace_bytes_varlen(const mdn_shape *shape, const int32_t *cu_seqlens, int32_t n_seq, int which, size_t *bytes_out) {
    Dims d;
    if (!bytes_out) return MDN_ERR_NULL;
    const int rc = check_varlen(shape, cu_seqlens, n_seq, &d);
    if (rc) return rc;
    if (which != MDN_WS_FWD && which != MDN_WS_BWD) return MDN_ERR_SHAPE;
    size_t need = 0;
    for (int i = 0; i < n_seq; ++i) {
        const int len = cu_seqlens[i + 1] - cu_seqlens[i];
        const Dims ds = seq_dims(d, len);
        // (a sequence run by itself may bring adjoints of its final states in)
        const size_t b = which == MDN_WS_FWD ? fwd_ws_total(ds, len % 64) : bwd_ws_total(ds, len % 64, ds.dtype == MDN_DTYPE_BF16);
        need = b > need ? b : need;
    }
    // (either way of running the batch may be taken: see mdn_chunk_fwd_varlen)
    size_t packed = carve_packed(d, cu_seqlens, n_seq, which == MDN_WS_BWD, nullptr).total;
    if (which == MDN_WS_FWD) {
        const size_t pf = carve_packed_final(d, cu_seqlens, n_seq, nullptr).total;
        packed = pf > packed ? pf : packed;
    }
    *bytes_out = packed > need ? packed : need;
    return MDN_OK;
}

int mdn_chunk_fwd_varlen(const mdn_shape *shape, const int32_t *cu_seqlens, int32_t n_seq, const void *q, const void *k,
                         const void *v, const float *beta, const float *alpha, const float *mu, const float *eta,
                         const float *S0, const float *M0, void *o, float *S_final, float *M_final, void *vt_saved,
                         void *workspace, size_t workspace_bytes, void *stream) {
    Dims d;
    int rc = check_varlen(shape, cu_seqlens, n_seq, &d);
    if (rc) return rc;
    if (!q || !k || !v || !beta || !alpha || !mu || !o || !workspace) return MDN_ERR_NULL;
    const void *ptrs[] = {q, k, v, beta, alpha, mu, eta, S0, M0, o, S_final, M_final, vt_saved, workspace};
    for (const void *p : ptrs)
        if (p && misaligned(p)) return MDN_ERR_ALIGN;
    size_t need = 0;
    rc = mdn_workspace_bytes_varlen(shape, cu_seqlens, n_seq, MDN_WS_FWD, &need);
    if (rc) return rc;
    if (workspace_bytes < need) return MDN_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!S0 && !M0 && !S_final && !M_final) {
        // no per-sequence states in or out: the batch as one stream of tokens
        const PackedWs w = carve_packed(d, cu_seqlens, n_seq, false, workspace);
        rc = packed_gates(d, cu_seqlens, n_seq, alpha, mu, w, s);
        if (rc) return rc;
        const size_t es = elem_size(d), rk = (size_t)d.H * d.dk * es, rv = (size_t)d.H * d.dv * es, rg = (size_t)d.H * 4;
        auto part = [&](size_t t0, int len, void *ws, hipStream_t st) {
            FwdCall c = {at_token(q, t0, rk), at_token(k, t0, rk), at_token(v, t0, rv), at_token(beta, t0, rg),
                         at_token(w.alpha, t0, rg), at_token(w.mu, t0, rg), at_token(eta, t0, rg), nullptr, nullptr,
                         at_token(o, t0, rv), nullptr, nullptr, at_token(vt_saved, t0, rv), nullptr, nullptr};
            return fwd_any(seq_dims(d, len), len % 64, c, ws, st);
        };
        if (!w.cut) return part(0, d.T, w.rest, s);
        const int t1 = cu_seqlens[w.cut];
        return run_beside(s, [&](hipStream_t st) { return part(0, t1, w.rest, st); },
                          [&](hipStream_t st) { return part((size_t)t1, d.T - t1, w.rest2, st); });
    }
    if (!S0 && !M0 && S_final && M_final) {
        // zero initial states, final states of every sequence wanted: the stream, then the sequences' last chunks
        const PackedFinalWs w = carve_packed_final(d, cu_seqlens, n_seq, workspace);
        rc = packed_gates(d, cu_seqlens, n_seq, alpha, mu, w.g, s);
        if (rc) return rc;
        const size_t es = elem_size(d), rk = (size_t)d.H * d.dk * es, rv = (size_t)d.H * d.dv * es, rg = (size_t)d.H * 4;
        auto part = [&](const StreamPiece &pc, hipStream_t st) {
            const size_t t0 = (size_t)pc.t0;
            FwdCall c = {at_token(q, t0, rk), at_token(k, t0, rk), at_token(v, t0, rv), at_token(beta, t0, rg),
                         at_token(w.g.alpha, t0, rg), at_token(w.g.mu, t0, rg), at_token(eta, t0, rg), nullptr, nullptr,
                         at_token(o, t0, rv), nullptr, nullptr, at_token(vt_saved, t0, rv), pc.states, nullptr, pc.states_lo};
            return fwd_any(seq_dims(d, pc.len), pc.len % 64, c, pc.rest, st);
        };
        rc = w.npieces == 1 ? part(w.piece[0], s)
                            : run_beside(s, [&](hipStream_t st) { return part(w.piece[0], st); },
                                         [&](hipStream_t st) { return part(w.piece[1], st); });
        if (rc) return rc;
        const FwdCall whole = {q, k, v, beta, w.g.alpha, w.g.mu, eta, nullptr, nullptr, o, nullptr, nullptr, vt_saved, nullptr,
                               nullptr};
        return packed_final_states(d, cu_seqlens, n_seq, whole, w, S_final, M_final, s);
    }
    const size_t es = elem_size(d), rk = (size_t)d.H * d.dk * es, rv = (size_t)d.H * d.dv * es, rg = (size_t)d.H * 4;
    const size_t st = (size_t)d.H * d.dk * d.dv * sizeof(float);
    for (int i = 0; i < n_seq; ++i) {
        const size_t t0 = (size_t)cu_seqlens[i];
        const int len = cu_seqlens[i + 1] - cu_seqlens[i];
        FwdCall c = {at_token(q, t0, rk), at_token(k, t0, rk), at_token(v, t0, rv), at_token(beta, t0, rg),
                     at_token(alpha, t0, rg), at_token(mu, t0, rg), at_token(eta, t0, rg), at_token(S0, i, st),
                     at_token(M0, i, st), at_token(o, t0, rv), at_token(S_final, i, st), at_token(M_final, i, st),
                     at_token(vt_saved, t0, rv), nullptr, nullptr};
        rc = fwd_any(seq_dims(d, len), len % 64, c, workspace, s);
        if (rc) return rc;
    }
    return MDN_OK;
}

int mdn_chunk_bwd_varlen(const mdn_shape *shape, const int32_t *cu_seqlens, int32_t n_seq, const void *q, const void *k,
                         const void *v, const float *beta, const float *alpha, const float *mu, const float *eta,
                         const float *S0, const float *M0, const void *vt_saved, const void *dO, const float *dS_final,
                         const float *dM_final, void *dq, void *dk, void *dv, float *dbeta, float *dalpha, float *dmu,
                         float *deta, float *dS0, float *dM0, void *workspace, size_t workspace_bytes, void *stream) {
    Dims d;
    int rc = check_varlen(shape, cu_seqlens, n_seq, &d);
    if (rc) return rc;
    if (!q || !k || !v || !beta || !alpha || !mu || !vt_saved || !dO || !dq || !dk || !dv || !dbeta || !dalpha || !dmu ||
        !workspace)
        return MDN_ERR_NULL;
    const void *ptrs[] = {q, k, v, beta, alpha, mu, eta, S0, M0, vt_saved, dO, dS_final, dM_final, dq, dk, dv, dbeta, dalpha,
                          dmu, deta, dS0, dM0, workspace};
    for (const void *p : ptrs)
        if (p && misaligned(p)) return MDN_ERR_ALIGN;
    size_t need = 0;
    rc = mdn_workspace_bytes_varlen(shape, cu_seqlens, n_seq, MDN_WS_BWD, &need);
    if (rc) return rc;
    if (workspace_bytes < need) return MDN_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!S0 && !M0 && !dS_final && !dM_final && !dS0 && !dM0) {
        // no per-sequence states or state adjoints in or out: the batch as one stream of tokens
        const PackedWs w = carve_packed(d, cu_seqlens, n_seq, true, workspace);
        rc = packed_gates(d, cu_seqlens, n_seq, alpha, mu, w, s);
        if (rc) return rc;
        const size_t es = elem_size(d), rk = (size_t)d.H * d.dk * es, rv = (size_t)d.H * d.dv * es, rg = (size_t)d.H * 4;
        auto part = [&](size_t t0, int len, void *ws, hipStream_t st) {
            BwdCall c = {at_token(q, t0, rk), at_token(k, t0, rk), at_token(v, t0, rv), at_token(beta, t0, rg),
                         at_token(w.alpha, t0, rg), at_token(w.mu, t0, rg), at_token(eta, t0, rg), nullptr, nullptr,
                         at_token(vt_saved, t0, rv), nullptr, nullptr, at_token(dO, t0, rv), nullptr, nullptr,
                         at_token(dq, t0, rk), at_token(dk, t0, rk), at_token(dv, t0, rv), at_token(dbeta, t0, rg),
                         at_token(dalpha, t0, rg), at_token(dmu, t0, rg), at_token(deta, t0, rg), nullptr, nullptr};
            return bwd_any(seq_dims(d, len), len % 64, c, ws, st);
        };
        if (!w.cut) {
            rc = part(0, d.T, w.rest, s);
        } else {
            const int t1 = cu_seqlens[w.cut];
            rc = run_beside(s, [&](hipStream_t st) { return part(0, t1, w.rest, st); },
                            [&](hipStream_t st) { return part((size_t)t1, d.T - t1, w.rest2, st); });
        }
        if (rc) return rc;
        return set_at_sequence_starts(d, cu_seqlens, n_seq, dalpha, dmu, 0.f, s);
    }
    const size_t es = elem_size(d), rk = (size_t)d.H * d.dk * es, rv = (size_t)d.H * d.dv * es, rg = (size_t)d.H * 4;
    const size_t st = (size_t)d.H * d.dk * d.dv * sizeof(float);
    for (int i = 0; i < n_seq; ++i) {
        const size_t t0 = (size_t)cu_seqlens[i];
        const int len = cu_seqlens[i + 1] - cu_seqlens[i];
        BwdCall c = {at_token(q, t0, rk), at_token(k, t0, rk), at_token(v, t0, rv), at_token(beta, t0, rg),
                     at_token(alpha, t0, rg), at_token(mu, t0, rg), at_token(eta, t0, rg), at_token(S0, i, st),
                     at_token(M0, i, st), at_token(vt_saved, t0, rv), nullptr, nullptr, at_token(dO, t0, rv),
                     at_token(dS_final, i, st), at_token(dM_final, i, st), at_token(dq, t0, rk), at_token(dk, t0, rk),
                     at_token(dv, t0, rv), at_token(dbeta, t0, rg), at_token(dalpha, t0, rg), at_token(dmu, t0, rg),
                     at_token(deta, t0, rg), at_token(dS0, i, st), at_token(dM0, i, st)};
        rc = bwd_any(seq_dims(d, len), len % 64, c, workspace, s);
        if (rc) return rc;
    }
    return MDN_OK;
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
