/*
 * C ABI of the MI355X (gfx950) Momentum DeltaNet (MDN) library.
 *
 * The operation is the stepwise-momentum delta rule of Sec. 3.1 (Eq. Mt.recurrent /
 * St.recurrent).  Per (batch b, head h), with states S, M in R^{dk x dv}:
 *
 *     p_t = alpha_t k_t                      v~_t = v_t - S_{t-1}^T p_t
 *     M_t = mu_t M_{t-1} - eta_t k_t v~_t^T  S_t  = alpha_t S_{t-1} - beta_t M_t
 *     o_t = scale * S_t^T q_t                (read-out of the post-update state)
 *
 * mdn_chunk_fwd / mdn_chunk_bwd evaluate it (and its reverse-mode adjoint) with the exact
 * chunkwise-parallel algorithm of Sec. 3.1 "Chunkwise Algorithm" / Appendix C-D;
 * mdn_recurrent_step evaluates it token by token (decoding, Appendix E recurrent form).
 *
 * Conventions shared by every entry point
 *   - Every pointer is a DEVICE pointer unless stated otherwise; the caller owns all buffers and
 *     the library allocates no device memory.  What it keeps between calls, all of it safe to use
 *     from several host threads: the mdn_set_segments() setting (one atomic integer for the
 *     process); the event list of the optional timing facility at the end of this header (behind a
 *     mutex); and, once a call has been split over two streams, one extra stream and a few events
 *     per device, shared by all calls on that device (a call that uses them holds the device's
 *     mutex while it enqueues, so concurrent callers are serialised on that second stream, never
 *     mixed up).
 *   - Token tensors are contiguous [B, T, H, D] (D = dk for q, k; dv for v, o), gates are
 *     contiguous [B, T, H] fp32 in the LINEAR domain (alpha, mu in [0,1], beta step size;
 *     mu = 0 is allowed), states are contiguous [B, H, dk, dv] fp32.
 *   - shape.dtype selects the storage type of q, k, v, o, dO, dq, dk, dv and of every
 *     intermediate the library stores: MDN_DTYPE_BF16 (bf16 MFMA operands, fp32 accumulation
 *     and fp32 states) or MDN_DTYPE_F32 (fp32 MFMA throughout).
 *   - All pointers must be 16-byte aligned.  dk, dv in {64, 128}; C in {16, 32, 64} (Algorithm 1's chunk sizes);
 *     any T >= 1: when T is not a multiple of C the last chunk is partial (Algorithm 1 pads it; here the padding
 *     tokens are exact identity steps, k = v = q = 0, alpha = mu = 1, beta = 0, on copies inside the workspace, so
 *     outputs, final states and gradients are those of the T tokens given).  C = 64 is the tuned path: the kernels
 *     work on 64-token tiles, and a chunk of 16 or 32 tokens runs as one such tile filled up with identity steps
 *     (the exact algorithm at that chunk size, at 64 / C times the work and workspace; results do not depend on C
 *     beyond rounding).  The packed variable-length calls take C = 64 only.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     ordered after what the stream already holds and is complete when the stream reaches the
 *     end of the call; no call synchronises.  When the serial scans would leave at least half
 *     of the GPU idle (few batch*head pairs, many chunks) mdn_chunk_fwd / mdn_chunk_bwd split
 *     the sequence into segments and run the chunk-parallel kernel of one segment beside the
 *     scan of its neighbour on a second stream that the library creates once per device
 *     (default priority) and joins back into `stream` with events, also when a launch fails on the
 *     way; see mdn_set_segments().
 *   - Return value: MDN_OK (0) or a negative MDN_ERR_* code; nothing is launched when an
 *     error is returned from validation.  NaN/Inf in the inputs propagate, they are not detected.
 *   - No environment variable or other hidden setting influences a call.
 */
#ifndef MDN_H
#define MDN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { MDN_DTYPE_BF16 = 0, MDN_DTYPE_F32 = 1 };

enum {
    MDN_OK = 0,
    MDN_ERR_NULL = -1,      /* a required pointer is NULL */
    MDN_ERR_SHAPE = -2,     /* unsupported B/T/H/dk/dv/C (dk or dv not in {64,128}, C not in {16,32,64}, sizes < 1, ...) */
    MDN_ERR_DTYPE = -3,     /* dtype is neither MDN_DTYPE_BF16 nor MDN_DTYPE_F32 */
    MDN_ERR_WORKSPACE = -4, /* workspace_bytes smaller than mdn_workspace_bytes() reports */
    MDN_ERR_ALIGN = -5,     /* a pointer is not 16-byte aligned */
    MDN_ERR_LAUNCH = -6,    /* a kernel launch failed (hipGetLastError) */
    MDN_ERR_DEVICE = -7     /* the current device is not a gfx950 GPU */
};

enum { MDN_WS_FWD = 0, MDN_WS_BWD = 1, MDN_WS_BWD_STATE_ADJOINTS = 2 };

typedef struct mdn_shape {
    int32_t B, T, H;  /* batch, sequence length, heads */
    int32_t dk, dv;   /* key / value head dimensions */
    int32_t C;        /* chunk size: 64 (the tuned path), 32 or 16; ignored by mdn_recurrent_step */
    int32_t dtype;    /* MDN_DTYPE_* */
    float scale;      /* multiplies q; the paper's default is dk^-1/2 (Appendix E) */
} mdn_shape;

/* Bytes of scratch `workspace` that mdn_chunk_fwd (which = MDN_WS_FWD) or mdn_chunk_bwd
 * (MDN_WS_BWD; MDN_WS_BWD_STATE_ADJOINTS for a call that passes dS_final or dM_final) needs for this shape.
 * Host-only; touches no device. */
int mdn_workspace_bytes(const mdn_shape *shape, int which, size_t *bytes_out);

/* Bytes of the optional `states_saved` buffer: the states S, M at the start of every chunk in the storage
 * dtype, 2 dk dv elements per (batch, head, chunk), ceil(T/C) chunks.  Only mdn_chunk_bwd reads it (the blocks
 * of the full chunks come first, [B, H, T/C, 2, dk, dv], then one block per (batch, head) for a partial chunk). */
int mdn_saved_states_bytes(const mdn_shape *shape, size_t *bytes_out);

/* Bytes of the optional `operands_saved` buffer: the chunk-local operands of the reverse pass
 * (transposed key and query tiles, masked products and triangular inverse, Sec. 3.1 "Chunkwise
 * Algorithm") that a training forward can keep so that the backward does not recompute them. */
int mdn_saved_operands_bytes(const mdn_shape *shape, size_t *bytes_out);

/*
 * Chunkwise forward (Sec. 3.1 "Chunkwise Algorithm"; Appendix C, D).
 *   in : q, k [B,T,H,dk], v [B,T,H,dv] (storage dtype); beta, alpha, mu [B,T,H] fp32;
 *        eta [B,T,H] fp32 or NULL (= 1); S0, M0 [B,H,dk,dv] fp32 or NULL (= 0).
 *   out: o [B,T,H,dv] (storage dtype);
 *        S_final, M_final [B,H,dk,dv] fp32, each may be NULL (not written);
 *        vt_saved [B,T,H,dv] (storage dtype) or NULL: the correction values V~ that
 *        mdn_chunk_bwd needs (Sec. 3.1 "Practical Considerations");
 *        states_saved (see mdn_saved_states_bytes) or NULL: chunk-start states; when given to
 *        mdn_chunk_bwd it skips their reconstruction from V~;
 *        operands_saved (see mdn_saved_operands_bytes) or NULL: chunk-local operands of the
 *        reverse pass; when given to mdn_chunk_bwd it skips their recomputation.
 *   workspace: at least mdn_workspace_bytes(MDN_WS_FWD); contents are scratch.
 */
int mdn_chunk_fwd(const mdn_shape *shape, const void *q, const void *k, const void *v, const float *beta,
                  const float *alpha, const float *mu, const float *eta, const float *S0, const float *M0,
                  void *o, float *S_final, float *M_final, void *vt_saved, void *states_saved,
                  void *operands_saved, void *workspace, size_t workspace_bytes, void *stream);

/*
 * mdn_chunk_fwd for callers that cannot allocate device memory or create streams and events: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs, results (bit for bit) and
 * errors as mdn_chunk_fwd without states_saved / operands_saved; what would be the workspace is a fixed array of
 * MDN_NOALLOC_SCRATCH_BYTES inside the library's device image (each GPU the library runs on holds its own copy until
 * the process ends).  The call allocates nothing, creates nothing and never uses a second stream (one launch sequence
 * on `stream`, whatever the shape).
 *   - A shape whose mdn_workspace_bytes(MDN_WS_FWD) exceeds MDN_NOALLOC_SCRATCH_BYTES is refused with
 *     MDN_ERR_WORKSPACE before anything is launched (16-bit storage, d = 128: about 18 KB per chunk and
 *     (batch, head) pair, i.e. up to B*H*T = 233 000 tokens-heads; 32-bit storage, d = 128: 66 KB per chunk).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two host
 *     threads) race on it and give wrong results; calls ordered on one stream are safe.  The array keeps the last
 *     call's contents; nothing in it has to start from zero.
 */
#define MDN_NOALLOC_SCRATCH_BYTES (64u << 20)
int mdn_chunk_fwd_noalloc(const mdn_shape *shape, const void *q, const void *k, const void *v, const float *beta,
                          const float *alpha, const float *mu, const float *eta, const float *S0, const float *M0,
                          void *o, float *S_final, float *M_final, void *vt_saved, void *stream);

/*
 * Chunkwise backward: adjoint of mdn_chunk_fwd for the scalar
 *     L = <o, dO> + <S_final, dS_final> + <M_final, dM_final>.
 * The forward keeps V~ only (Sec. 3.1 "Practical Considerations"); the chunk-start states
 * are reconstructed from it unless states_saved is given.
 *   in : the forward inputs (same pointers/values as in the forward call), vt_saved (required),
 *        states_saved or NULL, operands_saved or NULL, dO [B,T,H,dv] (storage dtype),
 *        dS_final, dM_final [B,H,dk,dv] fp32 or NULL (= 0).
 *   out: dq, dk [B,T,H,dk], dv [B,T,H,dv] (storage dtype); dbeta, dalpha, dmu [B,T,H] fp32;
 *        deta [B,T,H] fp32 or NULL; dS0, dM0 [B,H,dk,dv] fp32 or NULL.
 *        Gradients are with respect to the linear gate values.
 *   workspace: at least mdn_workspace_bytes(MDN_WS_BWD); with dS_final or dM_final given,
 *        mdn_workspace_bytes(MDN_WS_BWD_STATE_ADJOINTS).  Adjoints that enter from outside can be large against
 *        everything dO puts into the states, so with 16-bit storage such a call carries the chunk states and their
 *        adjoints between its kernels as bf16 pairs (value + rounding remainder) and reconstructs the states from
 *        V~ even when states_saved is given (the forward's copy has no remainders).
 */
int mdn_chunk_bwd(const mdn_shape *shape, const void *q, const void *k, const void *v, const float *beta,
                  const float *alpha, const float *mu, const float *eta, const float *S0, const float *M0,
                  const void *vt_saved, const void *states_saved, const void *operands_saved, const void *dO,
                  const float *dS_final, const float *dM_final, void *dq, void *dk, void *dv, float *dbeta, float *dalpha,
                  float *dmu, float *deta, float *dS0, float *dM0, void *workspace, size_t workspace_bytes,
                  void *stream);

/*
 * Packed variable-length batches (Algorithm 1 is per sequence; a training batch usually packs several): the
 * sequences lie one after another along T of [1, T, H, *] tensors, sequence i being the tokens
 * [cu_seqlens[i], cu_seqlens[i+1]); cu_seqlens is a HOST array of n_seq + 1 increasing offsets with cu_seqlens[0] = 0
 * and cu_seqlens[n_seq] = shape.T; shape.B must be 1.  States are [n_seq, H, dk, dv].  Any lengths >= 1.
 * A call that neither gives nor asks for per-sequence states (forward: S0, M0, S_final, M_final all NULL; backward:
 * S0, M0, dS_final, dM_final, dS0, dM0 all NULL) runs the whole batch as ONE stream of shape.T tokens, with alpha and
 * mu set to zero (in copies of its own) at the first token of every sequence but the first: by Eq. Mt.recurrent /
 * St.recurrent such a token neither sees the states before it nor passes an adjoint back to them, which is what a
 * sequence that starts from zero states computes; the gradients of those zeroed gates are zero.  One set of
 * launches however many the sequences.  A forward with zero initial states that wants the final states (S0, M0 NULL,
 * S_final and M_final given: prefill of a batch of prompts) runs the same stream, keeps its chunk-start states in the
 * workspace and then runs, as one batch, the last chunk of every sequence once more from its start state up to the
 * sequence's end (with 16-bit storage the start states are kept as value + rounding remainder, so the final states
 * start from fp32-accurate states as in mdn_chunk_fwd).  Any other call runs each
 * sequence by itself through the same kernels as
 * mdn_chunk_fwd / mdn_chunk_bwd, one after the other on the stream (exact, but a batch of many short sequences does
 * not fill the GPU).  The backward reconstructs the states and recomputes the operands (no states_saved /
 * operands_saved here).  workspace: mdn_workspace_bytes_varlen.
 * Errors as for the fixed-length calls; MDN_ERR_SHAPE also for inconsistent cu_seqlens.
 */
int mdn_workspace_bytes_varlen(const mdn_shape *shape, const int32_t *cu_seqlens, int32_t n_seq, int which, size_t *bytes_out);
int mdn_chunk_fwd_varlen(const mdn_shape *shape, const int32_t *cu_seqlens, int32_t n_seq, const void *q, const void *k,
                         const void *v, const float *beta, const float *alpha, const float *mu, const float *eta,
                         const float *S0, const float *M0, void *o, float *S_final, float *M_final, void *vt_saved,
                         void *workspace, size_t workspace_bytes, void *stream);
int mdn_chunk_bwd_varlen(const mdn_shape *shape, const int32_t *cu_seqlens, int32_t n_seq, const void *q, const void *k,
                         const void *v, const float *beta, const float *alpha, const float *mu, const float *eta,
                         const float *S0, const float *M0, const void *vt_saved, const void *dO, const float *dS_final,
                         const float *dM_final, void *dq, void *dk, void *dv, float *dbeta, float *dalpha, float *dmu,
                         float *deta, float *dS0, float *dM0, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Recurrent (decoding) form, Eq. Mt.recurrent / St.recurrent, Appendix E recurrent form:
 * advances S, M in place over the shape.T tokens given (usually T = 1) and writes o.
 *   in : q, k, v, beta, alpha, mu, eta as for mdn_chunk_fwd (T tokens);
 *   io : S, M [B,H,dk,dv] fp32, updated in place;
 *   out: o [B,T,H,dv] (storage dtype).
 * No chunk-size restriction on T (T >= 1).
 */
int mdn_recurrent_step(const mdn_shape *shape, const void *q, const void *k, const void *v, const float *beta,
                       const float *alpha, const float *mu, const float *eta, float *S, float *M, void *o,
                       void *stream);

/*
 * Stability-aware gate parameterisation (Sec. 3.3, "Stability Aware Gating Parameterization"): from the four
 * per-head projections of every token to the linear-domain gates that mdn_chunk_fwd / mdn_recurrent_step take,
 *     eta   = tanh(x_eta / tau) + 1,    theta = arctan(eta s),   alpha_max = cos^2 theta,   beta_max = sin^2 theta,
 *     alpha = alpha_max exp(-a_alpha[h] softplus(x_alpha + b_alpha[h])),
 *     mu    = exp(max(-a_mu[h] softplus(x_mu + b_mu[h]), mu_log_min)),        beta = sigmoid(x_beta) beta_max.
 * All tensors [B,T,H] fp32 contiguous on the device; a_alpha, b_alpha, a_mu, b_mu are device vectors of H floats
 * (the caller's; a_* > 0); s, tau > 0 and mu_log_min (the paper's default -1) are host scalars.
 * mdn_gates_bwd is the adjoint for L = <alpha,dalpha> + <beta,dbeta> + <mu,dmu> + <eta,deta> (the four gradients
 * that mdn_chunk_bwd returns): dx_* [B,T,H], and dparams = [4][H] floats (da_alpha, db_alpha, da_mu, db_mu;
 * overwritten; summed with floating-point atomics, so the last bits depend on the order) or NULL.
 * Errors: MDN_ERR_NULL, MDN_ERR_SHAPE (sizes < 1, H > 1024, tau <= 0), MDN_ERR_LAUNCH.  Nothing is allocated.
 */
typedef struct mdn_gate_params {
    int32_t B, T, H;
    const float *a_alpha, *b_alpha, *a_mu, *b_mu; /* device, [H] each */
    float s, tau, mu_log_min;
} mdn_gate_params;

int mdn_gates_fwd(const mdn_gate_params *params, const float *x_alpha, const float *x_mu, const float *x_beta,
                  const float *x_eta, float *alpha, float *beta, float *mu, float *eta, void *stream);
int mdn_gates_bwd(const mdn_gate_params *params, const float *x_alpha, const float *x_mu, const float *x_beta,
                  const float *x_eta, const float *dalpha, const float *dbeta, const float *dmu, const float *deta,
                  float *dx_alpha, float *dx_mu, float *dx_beta, float *dx_eta, float *dparams, void *stream);

/*
 * The elementwise operations around the delta rule in the MDN layer (Sec. 3.3, architecture paragraph) and their
 * adjoints.  shape gives B, T, H, dk = dv in {64, 128} and the storage dtype of the [B,T,H,d] tensors (C and scale
 * are not used); parameter vectors are device fp32; eps is the constant under the square roots.
 *   front end, on the short-convolution outputs x_q, x_k [B,T,H,dk], x_v [B,T,H,dv], with d [H]:
 *       q = L2Norm(SiLU(x_q) - d_h SiLU(x_k))   (output correction, applied before the normalisation),
 *       k = L2Norm(SiLU(x_k)),   v = SiLU(x_v),   L2Norm(x) = x / sqrt(sum x^2 + eps);
 *     mdn_frontend_bwd: dq, dk, dv -> dx_q, dx_k, dx_v and dd [H] (overwritten; NULL = not wanted).
 *   back end, on the output o of the delta rule and the gate projection g, both [B,T,H,dv], with w [dv]:
 *       y = sigmoid(g) * w * o / sqrt(mean(o^2) + eps)   (head-wise RMS norm, data-dependent output gate);
 *     mdn_epilogue_bwd: dy -> d_o, dg and dw [dv] (overwritten; NULL = not wanted).
 * Parameter gradients are summed with floating-point atomics (last bits depend on the order).  Nothing is allocated.
 * Errors: MDN_ERR_NULL, MDN_ERR_SHAPE, MDN_ERR_DTYPE, MDN_ERR_LAUNCH.
 */
int mdn_frontend_fwd(const mdn_shape *shape, const void *x_q, const void *x_k, const void *x_v, const float *d, float eps,
                     void *q, void *k, void *v, void *stream);
int mdn_frontend_bwd(const mdn_shape *shape, const void *x_q, const void *x_k, const void *x_v, const float *d, float eps,
                     const void *dq, const void *dk, const void *dv, void *dx_q, void *dx_k, void *dx_v, float *dd,
                     void *stream);
int mdn_epilogue_fwd(const mdn_shape *shape, const void *o, const void *g, const float *w, float eps, void *y, void *stream);
int mdn_epilogue_bwd(const mdn_shape *shape, const void *o, const void *g, const float *w, float eps, const void *dy,
                     void *d_o, void *dg, float *dw, void *stream);

/*
 * Optional per-kernel timing (used by the benchmark to attribute time to kernels).
 * Between mdn_profile_begin() and mdn_profile_end() every kernel the library launches is
 * bracketed by a pair of HIP events recorded on the launch stream.  mdn_profile_end()
 * synchronises those events and adds, per kernel id, the elapsed milliseconds into ms[id] and
 * the number of launches into launches[id] (HOST arrays of n entries; ids >= n are dropped),
 * then releases the events.  The switch is process-wide (launches of every thread are recorded while it is
 * on); meant for one benchmarking thread.
 */
enum {
    MDN_KERNEL_INTRA_FWD = 0, /* chunk-local coefficients, masked products, triangular solve
                                 (and the reverse pass's operands when operands_saved is given) */
    MDN_KERNEL_SCAN_FWD = 1,  /* sequential inter-chunk propagation of S and M, outputs */
    MDN_KERNEL_INTRA_BWD = 2, /* same as 0 in the operand layouts of the reverse pass */
    MDN_KERNEL_REBUILD = 3,   /* chunk-start states reconstructed from V~ */
    MDN_KERNEL_SCAN_BWD = 4,  /* reverse inter-chunk scan of dS, dM */
    MDN_KERNEL_GRAD = 5,      /* chunk-parallel gradients dq, dk, dv, dalpha, dbeta, dmu, deta */
    MDN_KERNEL_RECURRENT = 6, /* token-by-token recurrent form */
    MDN_KERNEL_COUNT = 7
};
int mdn_profile_begin(void);
int mdn_profile_end(float *ms, int *launches, int n);
/* An event pair costs a few microseconds of GPU time (the next launch waits for the marker in front of it), so a
 * benchmark that wants kernel durations out of its timed region without paying for a pair around every launch brackets
 * only every period-th launch of the library (period >= 1; mdn_profile_begin() = period 1): with a period that shares no
 * factor with the number of launches per step, the bracketed launch walks through the kernels step after step.
 * mdn_profile_end() then returns the bracketed launches; mdn_profile_launch_counts() the number of ALL launches per kernel id
 * since the last begin (host array of n entries; call it before or after mdn_profile_end). */
int mdn_profile_begin_sampled(int period);
int mdn_profile_launch_counts(int *launched, int n);

/*
 * Number of segments mdn_chunk_fwd / mdn_chunk_bwd split the sequence into: k >= 1 forces k
 * (1 = never split; capped at N/4 and at 16), 0 restores the automatic choice.  A tuning and
 * test knob: results do not depend on it (states cross a segment boundary in fp32, exactly as
 * they are carried inside a scan).  Returns the previous setting (an atomic exchange: process-wide).
 */
int mdn_set_segments(int k);

/* Static, human-readable text for a return code. */
const char *mdn_strerror(int code);

/* Library version (major * 100 + minor). */
int mdn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MDN_H */
