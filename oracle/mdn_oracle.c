/*
 * Momentum DeltaNet (MDN) reference oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, token-by-token fp64 CPU implementation of the stepwise-momentum
 * delta rule exactly as the paper defines it (Sec. 3.1, Eq. "Mt.recurrent" /
 * "St.recurrent", the definition of the correction value v~ and of p = alpha*k in
 * the paragraph below them; Appendix E, recurrent form, fixes the order of the
 * operations and where `scale` is applied).  Nothing here is blocked, fused or
 * reordered: one token at a time, one (batch, head) pair at a time.
 *
 * Only tests, the smoke check and the cpu_baseline leg of the benchmark may call
 * this file.  The GPU library shares no code with it.
 *
 * Per (b, h), with S, M in R^{dk x dv} (row-major [dk][dv]):
 *     p_t  = alpha_t k_t
 *     e_t  = v_t - S_{t-1}^T p_t                      (correction value v~_t)
 *     M_t  = mu_t M_{t-1} - eta_t k_t e_t^T
 *     S_t  = alpha_t S_{t-1} - beta_t M_t
 *     o_t  = scale * S_t^T q_t                        (reads the POST-update state)
 *
 * The gradient oracle is the hand-derived token-level reverse-mode adjoint of these
 * five lines (the paper prints no backward equations).  It is pinned in the tests by
 * central finite differences of the forward and by an independent autograd run.
 *
 * Layouts (all contiguous, double):  q,k [B,T,H,dk];  v,o [B,T,H,dv];
 * alpha,beta,mu,eta [B,T,H];  states [B,H,dk,dv].  eta == NULL means eta = 1;
 * S0/M0 == NULL means zero initial state.
 *
 * Pins: every function here is pinned (see tests/test_oracle_pins.py); the paper
 * prints no worked numeric example, so absolute values are pinned through closed
 * forms, special cases, brute force and finite differences only.
 */
#include <stdlib.h>
#include <string.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int B, T, H, dk, dv;
    double scale;
    const double *q, *k, *v, *alpha, *beta, *mu, *eta, *S0, *M0;
} mdn_oracle_in;

static size_t tok_off(const mdn_oracle_in *in, int b, int t, int h) {
    return ((size_t)b * in->T + t) * in->H + h;
}

/* One token of the recurrence, in place on S and M.  e (length dv) receives v~_t. */
static void step_token(int dk, int dv, const double *k, const double *v, double alpha, double beta,
                       double mu, double eta, double *S, double *M, double *e) {
    /* e = v - S^T (alpha k) */
    for (int j = 0; j < dv; ++j) e[j] = v[j];
    for (int i = 0; i < dk; ++i) {
        double p = alpha * k[i];
        const double *Si = S + (size_t)i * dv;
        for (int j = 0; j < dv; ++j) e[j] -= p * Si[j];
    }
    /* M = mu M - eta k e^T ;  S = alpha S - beta M */
    for (int i = 0; i < dk; ++i) {
        double ek = eta * k[i];
        double *Mi = M + (size_t)i * dv;
        double *Si = S + (size_t)i * dv;
        for (int j = 0; j < dv; ++j) {
            Mi[j] = mu * Mi[j] - ek * e[j];
            Si[j] = alpha * Si[j] - beta * Mi[j];
        }
    }
}

static void read_out(int dk, int dv, double scale, const double *q, const double *S, double *o) {
    for (int j = 0; j < dv; ++j) o[j] = 0.0;
    for (int i = 0; i < dk; ++i) {
        double qi = scale * q[i];
        const double *Si = S + (size_t)i * dv;
        for (int j = 0; j < dv; ++j) o[j] += qi * Si[j];
    }
}

static void init_state(const double *src, size_t bh, size_t n, double *dst) {
    if (src) memcpy(dst, src + bh * n, n * sizeof(double));
    else memset(dst, 0, n * sizeof(double));
}

/* Forward.  o is required; S_out / M_out / vt_out (the correction values, [B,T,H,dv]) may be NULL.
 * Returns the number of threads used, or a negative value on allocation failure. */
int mdn_oracle_forward(int B, int T, int H, int dk, int dv, double scale, const double *q, const double *k,
                       const double *v, const double *alpha, const double *beta, const double *mu,
                       const double *eta, const double *S0, const double *M0, double *o, double *S_out,
                       double *M_out, double *vt_out, int nthreads) {
    mdn_oracle_in in = {B, T, H, dk, dv, scale, q, k, v, alpha, beta, mu, eta, S0, M0};
    const size_t n = (size_t)dk * dv;
    int used = 1, fail = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#else
    (void)nthreads;
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * H; ++bh) {
        int b = bh / H, h = bh % H;
        double *S = (double *)malloc(n * sizeof(double));
        double *M = (double *)malloc(n * sizeof(double));
        double *e = (double *)malloc((size_t)dv * sizeof(double));
        if (!S || !M || !e) {
#pragma omp atomic write
            fail = 1;
        } else {
            init_state(in.S0, (size_t)bh, n, S);
            init_state(in.M0, (size_t)bh, n, M);
            for (int t = 0; t < T; ++t) {
                size_t g = tok_off(&in, b, t, h);
                double et = eta ? eta[g] : 1.0;
                step_token(dk, dv, k + g * dk, v + g * dv, alpha[g], beta[g], mu[g], et, S, M, e);
                read_out(dk, dv, scale, q + g * dk, S, o + g * dv);
                if (vt_out) memcpy(vt_out + g * dv, e, (size_t)dv * sizeof(double));
            }
            if (S_out) memcpy(S_out + (size_t)bh * n, S, n * sizeof(double));
            if (M_out) memcpy(M_out + (size_t)bh * n, M, n * sizeof(double));
        }
        free(S); free(M); free(e);
    }
    return fail ? -1 : used;
}

static double dot(const double *a, const double *b, size_t n) {
    double s = 0.0;
    for (size_t i = 0; i < n; ++i) s += a[i] * b[i];
    return s;
}

/*
 * Backward: token-level adjoint.  Given dO [B,T,H,dv] and optional adjoints of the final
 * states dS_T, dM_T [B,H,dk,dv], returns dq, dk, dv, dalpha, dbeta, dmu, deta (deta may be
 * NULL) and dS0, dM0 (may be NULL).
 *
 * The forward states are checkpointed every `seg` tokens; each segment is replayed to get
 * S_{t-1}, M_{t-1}, M_t, S_t, e_t for its tokens, then walked backwards:
 *
 *   o_t = scale S_t^T q_t        : dS += scale q_t dO_t^T ;  dq_t = scale S_t dO_t
 *   S_t = alpha S_{t-1} - beta M_t: dalpha += <dS,S_{t-1}> ; dbeta = -<dS,M_t> ; dM -= beta dS ; dSp = alpha dS
 *   M_t = mu M_{t-1} - eta k e^T : dmu = <dM,M_{t-1}> ; g = dM e ; deta = -k.g ; dk = -eta g ;
 *                                  de = -eta dM^T k ; dMp = mu dM
 *   e_t = v_t - S_{t-1}^T p      : dv_t = de ; dSp -= p de^T ; dp = -S_{t-1} de
 *   p   = alpha k                : dalpha += dp.k ; dk += alpha dp
 */
int mdn_oracle_backward(int B, int T, int H, int dk, int dv, double scale, const double *q, const double *k,
                        const double *v, const double *alpha, const double *beta, const double *mu,
                        const double *eta, const double *S0, const double *M0, const double *dO,
                        const double *dS_T, const double *dM_T, double *dq, double *dk_out, double *dv_out,
                        double *dalpha, double *dbeta, double *dmu, double *deta, double *dS0, double *dM0,
                        int nthreads) {
    mdn_oracle_in in = {B, T, H, dk, dv, scale, q, k, v, alpha, beta, mu, eta, S0, M0};
    const size_t n = (size_t)dk * dv;
    const int seg = 64;
    const int nseg = (T + seg - 1) / seg;
    int used = 1, fail = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#else
    (void)nthreads;
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * H; ++bh) {
        int b = bh / H, h = bh % H;
        /* checkpoints: state BEFORE the first token of each segment */
        double *ckS = (double *)malloc((size_t)nseg * n * sizeof(double));
        double *ckM = (double *)malloc((size_t)nseg * n * sizeof(double));
        /* per-segment replay: states after token i of the segment live at slot i+1; slot 0 = before */
        double *Ss = (double *)malloc((size_t)(seg + 1) * n * sizeof(double));
        double *Ms = (double *)malloc((size_t)(seg + 1) * n * sizeof(double));
        double *es = (double *)malloc((size_t)seg * dv * sizeof(double));
        double *dS = (double *)malloc(n * sizeof(double));
        double *dM = (double *)malloc(n * sizeof(double));
        double *g = (double *)malloc((size_t)dk * sizeof(double));
        double *de = (double *)malloc((size_t)dv * sizeof(double));
        if (!ckS || !ckM || !Ss || !Ms || !es || !dS || !dM || !g || !de) {
#pragma omp atomic write
            fail = 1;
        } else {
            /* pass 1: forward, keeping one checkpoint per segment */
            init_state(in.S0, (size_t)bh, n, Ss);
            init_state(in.M0, (size_t)bh, n, Ms);
            for (int t = 0; t < T; ++t) {
                if (t % seg == 0) {
                    memcpy(ckS + (size_t)(t / seg) * n, Ss, n * sizeof(double));
                    memcpy(ckM + (size_t)(t / seg) * n, Ms, n * sizeof(double));
                }
                size_t go = tok_off(&in, b, t, h);
                double et = eta ? eta[go] : 1.0;
                step_token(dk, dv, k + go * dk, v + go * dv, alpha[go], beta[go], mu[go], et, Ss, Ms, es);
            }
            init_state(dS_T, (size_t)bh, n, dS);
            init_state(dM_T, (size_t)bh, n, dM);
            /* pass 2: segments in reverse */
            for (int s = nseg - 1; s >= 0; --s) {
                int t0 = s * seg, len = (T - t0 < seg) ? (T - t0) : seg;
                memcpy(Ss, ckS + (size_t)s * n, n * sizeof(double));
                memcpy(Ms, ckM + (size_t)s * n, n * sizeof(double));
                for (int i = 0; i < len; ++i) {
                    size_t go = tok_off(&in, b, t0 + i, h);
                    double et = eta ? eta[go] : 1.0;
                    memcpy(Ss + (size_t)(i + 1) * n, Ss + (size_t)i * n, n * sizeof(double));
                    memcpy(Ms + (size_t)(i + 1) * n, Ms + (size_t)i * n, n * sizeof(double));
                    step_token(dk, dv, k + go * dk, v + go * dv, alpha[go], beta[go], mu[go], et,
                               Ss + (size_t)(i + 1) * n, Ms + (size_t)(i + 1) * n, es + (size_t)i * dv);
                }
                for (int i = len - 1; i >= 0; --i) {
                    size_t go = tok_off(&in, b, t0 + i, h);
                    const double *kt = k + go * dk, *qt = q + go * dk, *dOt = dO + go * dv;
                    const double *Sp = Ss + (size_t)i * n, *Mp = Ms + (size_t)i * n;
                    const double *St = Ss + (size_t)(i + 1) * n, *Mt = Ms + (size_t)(i + 1) * n;
                    const double *e = es + (size_t)i * dv;
                    double al = alpha[go], be = beta[go], m_ = mu[go], et = eta ? eta[go] : 1.0;
                    double *dqt = dq + go * dk, *dkt = dk_out + go * dk, *dvt = dv_out + go * dv;
                    /* read-out */
                    for (int a = 0; a < dk; ++a) {
                        double qa = scale * qt[a];
                        double *dSa = dS + (size_t)a * dv;
                        for (int j = 0; j < dv; ++j) dSa[j] += qa * dOt[j];
                        dqt[a] = scale * dot(St + (size_t)a * dv, dOt, (size_t)dv);
                    }
                    /* S_t = alpha S_{t-1} - beta M_t */
                    double dal = dot(dS, Sp, n);
                    dbeta[go] = -dot(dS, Mt, n);
                    for (size_t x = 0; x < n; ++x) dM[x] -= be * dS[x];
                    /* M_t = mu M_{t-1} - eta k e^T */
                    dmu[go] = dot(dM, Mp, n);
                    for (int a = 0; a < dk; ++a) g[a] = dot(dM + (size_t)a * dv, e, (size_t)dv);
                    double dn = 0.0;
                    for (int a = 0; a < dk; ++a) dn -= kt[a] * g[a];
                    if (deta) deta[go] = dn;
                    for (int a = 0; a < dk; ++a) dkt[a] = -et * g[a];
                    for (int j = 0; j < dv; ++j) de[j] = 0.0;
                    for (int a = 0; a < dk; ++a) {
                        double c = -et * kt[a];
                        const double *dMa = dM + (size_t)a * dv;
                        for (int j = 0; j < dv; ++j) de[j] += c * dMa[j];
                    }
                    /* propagate to the previous token's adjoints */
                    for (size_t x = 0; x < n; ++x) { dS[x] *= al; dM[x] *= m_; }
                    /* e = v - S_{t-1}^T p,  p = alpha k */
                    for (int j = 0; j < dv; ++j) dvt[j] = de[j];
                    for (int a = 0; a < dk; ++a) {
                        double pa = al * kt[a];
                        double *dSa = dS + (size_t)a * dv;
                        for (int j = 0; j < dv; ++j) dSa[j] -= pa * de[j];
                        double dpa = -dot(Sp + (size_t)a * dv, de, (size_t)dv);
                        dal += dpa * kt[a];
                        dkt[a] += al * dpa;
                    }
                    dalpha[go] = dal;
                }
            }
            if (dS0) memcpy(dS0 + (size_t)bh * n, dS, n * sizeof(double));
            if (dM0) memcpy(dM0 + (size_t)bh * n, dM, n * sizeof(double));
        }
        free(ckS); free(ckM); free(Ss); free(Ms); free(es); free(dS); free(dM); free(g); free(de);
    }
    return fail ? -1 : used;
}
