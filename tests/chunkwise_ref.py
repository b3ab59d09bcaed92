"""fp64 numpy statement of the paper's CHUNKWISE algorithm (Sec. 3.1 "Chunkwise Algorithm",
Appendix C/D) for one head, used only by the CPU tests:

* as a structurally different second implementation that pins the token-by-token oracle
  (dense inverse, Gamma from its definition (a_i/m_j)(c_i - c_{j-1}));
* as an executable statement of the chunk-level backward formulas (derived here; the paper
  prints none), checked against the oracle's token-level adjoint.

It shares no code with the oracle or with the GPU library.
Index convention: chunk-local i, j = 0..C-1; a, m, b, c are the inclusive prefix quantities.
"""
import numpy as np


def coeffs_def(alpha, beta, mu):
    """Eq. (coefficients): a = cumprod(alpha), m = cumprod(mu), c = cumsum(beta m / a), b = a c,
    Gamma_ij = (a_i/m_j)(c_i - c_{j-1}) for i >= j, Rho_ij = m_i/m_j.  Needs mu != 0."""
    a = np.cumprod(alpha)
    m = np.cumprod(mu)
    c = np.cumsum(beta * m / a)
    b = a * c
    cprev = np.concatenate([[0.0], c[:-1]])
    Gam = np.tril((a[:, None] / m[None, :]) * (c[:, None] - cprev[None, :]))
    Rho = np.tril(m[:, None] / m[None, :])
    return a, m, b, Gam, Rho


def coeffs_scan(alpha, beta, mu):
    """Division-free form of the same coefficients (valid at mu = 0 as well):
    Rho_jj = 1, Rho_ij = mu_i Rho_{i-1,j};  Gamma_ij = alpha_i Gamma_{i-1,j} + beta_i Rho_ij;
    b_i = alpha_i b_{i-1} + beta_i m_i."""
    C = len(alpha)
    a = np.cumprod(alpha)
    m = np.cumprod(mu)
    b = np.zeros(C)
    Gam = np.zeros((C, C))
    Rho = np.zeros((C, C))
    for i in range(C):
        b[i] = alpha[i] * (b[i - 1] if i else 0.0) + beta[i] * m[i]
        Rho[i, i] = 1.0
        if i:
            Rho[i, :i] = mu[i] * Rho[i - 1, :i]
            Gam[i, :i] = alpha[i] * Gam[i - 1, :i]
        Gam[i, : i + 1] += beta[i] * Rho[i, : i + 1]
    return a, m, b, Gam, Rho


def _shift_down(X):
    Y = np.zeros_like(X)
    Y[1:] = X[:-1]
    return Y


def chunk_pieces(q, k, v, alpha, beta, mu, eta, scale, coeffs=coeffs_def):
    """Everything of one chunk that does not depend on the incoming states."""
    a, m, b, Gam, Rho = coeffs(alpha, beta, mu)
    Kt = eta[:, None] * k          # K~ = diag(eta) K
    P = alpha[:, None] * k         # P  = diag(alpha) K
    Qs = scale * q
    am = np.concatenate([[1.0], a[:-1]])   # a^- (a_0 = 1)
    bm = np.concatenate([[0.0], b[:-1]])   # b^- (b_0 = 0)
    Gm = _shift_down(Gam)                  # Gamma^-_ij = Gamma_{i-1,j}
    A = (P @ Kt.T) * Gm                    # strictly lower triangular
    Tm = np.linalg.inv(np.eye(len(a)) + A)
    Bm = (Qs @ Kt.T) * Gam                 # lower triangular incl. diagonal (Gamma_ii = beta_i)
    return dict(a=a, m=m, b=b, Gam=Gam, Rho=Rho, Kt=Kt, P=P, Qs=Qs, am=am, bm=bm, Gm=Gm, A=A, T=Tm, Bm=Bm)


def forward(q, k, v, alpha, beta, mu, eta, S0, M0, scale, C, coeffs=coeffs_def):
    """One head: q,k [T,dk], v [T,dv], gates [T].  Returns o, S_T, M_T, v~, per-chunk start states."""
    T = q.shape[0]
    assert T % C == 0
    S, M = S0.copy(), M0.copy()
    o = np.zeros_like(v)
    vt = np.zeros_like(v)
    starts = []
    for n in range(T // C):
        sl = slice(n * C, (n + 1) * C)
        pc = chunk_pieces(q[sl], k[sl], v[sl], alpha[sl], beta[sl], mu[sl], eta[sl], scale, coeffs)
        starts.append((S.copy(), M.copy()))
        U = pc["T"] @ v[sl]
        Y = pc["T"] @ (pc["am"][:, None] * pc["P"])
        Z = pc["T"] @ (pc["bm"][:, None] * pc["P"])
        Vt = U - Y @ S + Z @ M
        o[sl] = pc["a"][:, None] * (pc["Qs"] @ S) - pc["b"][:, None] * (pc["Qs"] @ M) + pc["Bm"] @ Vt
        Sn = pc["a"][-1] * S - pc["b"][-1] * M + (pc["Gam"][-1][:, None] * pc["Kt"]).T @ Vt
        Mn = pc["m"][-1] * M - (pc["Rho"][-1][:, None] * pc["Kt"]).T @ Vt
        S, M = Sn, Mn
        vt[sl] = Vt
    return o, S, M, vt, starts


def backward(q, k, v, alpha, beta, mu, eta, S0, M0, scale, C, dO, dS_T, dM_T):
    """Chunk-level reverse pass for one head.  Returns dq, dk, dv, dalpha, dbeta, dmu, deta, dS0, dM0."""
    T, dk = q.shape
    N = T // C
    o, _, _, vt, starts = forward(q, k, v, alpha, beta, mu, eta, S0, M0, scale, C, coeffs_scan)
    dq = np.zeros_like(q); dkk = np.zeros_like(k); dv = np.zeros_like(v)
    dal = np.zeros(T); dbe = np.zeros(T); dmu = np.zeros(T); det = np.zeros(T)
    dS, dM = dS_T.copy(), dM_T.copy()          # adjoints of the state AFTER the current chunk
    for n in range(N - 1, -1, -1):
        sl = slice(n * C, (n + 1) * C)
        al, be, mm, et = alpha[sl], beta[sl], mu[sl], eta[sl]
        pc = chunk_pieces(q[sl], k[sl], v[sl], al, be, mm, et, scale, coeffs_scan)
        S, M = starts[n]
        Vt, dOc = vt[sl], dO[sl]
        a, m, b, Gam, Rho = pc["a"], pc["m"], pc["b"], pc["Gam"], pc["Rho"]
        Kt, P, Qs, am, bm, Gm, Tm, Bm = (pc[x] for x in ("Kt", "P", "Qs", "am", "bm", "Gm", "T", "Bm"))
        gC, rC = Gam[-1], Rho[-1]
        # --- serial part (reverse inter-chunk scan) ---
        dVt = Bm.T @ dOc + (gC[:, None] * Kt) @ dS - (rC[:, None] * Kt) @ dM
        dR = Tm.T @ dVt                                     # adjoint of the right-hand side; = dV
        dS_in = a[-1] * dS + (a[:, None] * Qs).T @ dOc - (am[:, None] * P).T @ dR
        dM_in = m[-1] * dM - b[-1] * dS - (b[:, None] * Qs).T @ dOc + (bm[:, None] * P).T @ dR
        # --- chunk-parallel part ---
        dv[sl] = dR
        dBm = np.tril(dOc @ Vt.T)
        dA = -np.tril(dR @ Vt.T, -1)
        W1 = dBm * Gam
        W2 = dA * Gm
        dOS, dOM = dOc @ S.T, dOc @ M.T
        dRS, dRM = dR @ S.T, dR @ M.T
        VdS, VdM = Vt @ dS.T, Vt @ dM.T
        dQs = W1 @ Kt + a[:, None] * dOS - b[:, None] * dOM
        dKt = W1.T @ Qs + W2.T @ P + gC[:, None] * VdS - rC[:, None] * VdM
        dP = W2 @ Kt - am[:, None] * dRS + bm[:, None] * dRM
        dq[sl] = scale * dQs
        dkk[sl] = et[:, None] * dKt + al[:, None] * dP
        det[sl] = (k[sl] * dKt).sum(1)
        dal_c = (k[sl] * dP).sum(1)
        # coefficient adjoints
        da = (dOS * Qs).sum(1); db = -(dOM * Qs).sum(1)
        dam = -(dRS * P).sum(1); dbm = (dRM * P).sum(1)
        da[-1] += (dS * S).sum(); db[-1] -= (dS * M).sum()
        dm = np.zeros(C); dm[-1] = (dM * M).sum()
        dGam = dBm * (Qs @ Kt.T)
        dGm = dA * (P @ Kt.T)
        dGam[:-1] += dGm[1:]                                # Gamma^-_ij = Gamma_{i-1,j}
        dGam[-1] += (VdS * Kt).sum(1)
        dRho = np.zeros((C, C)); dRho[-1] -= (VdM * Kt).sum(1)
        da[:-1] += dam[1:]; db[:-1] += dbm[1:]              # a^-_i = a_{i-1}, b^-_i = b_{i-1}
        dbe_c = np.zeros(C); dmu_c = np.zeros(C)
        for i in range(C - 1, -1, -1):
            # Gamma_ij = alpha_i Gamma_{i-1,j} + beta_i Rho_ij   (j <= i; Gamma_{i-1,i} = 0)
            if i:
                dal_c[i] += (dGam[i, :i] * Gam[i - 1, :i]).sum()
                dGam[i - 1, :i] += al[i] * dGam[i, :i]
            dbe_c[i] += (dGam[i, : i + 1] * Rho[i, : i + 1]).sum()
            dRho[i, : i + 1] += be[i] * dGam[i, : i + 1]
            # Rho_ij = mu_i Rho_{i-1,j}  (j < i)
            if i:
                dmu_c[i] += (dRho[i, :i] * Rho[i - 1, :i]).sum()
                dRho[i - 1, :i] += mm[i] * dRho[i, :i]
            # b_i = alpha_i b_{i-1} + beta_i m_i
            dal_c[i] += db[i] * (b[i - 1] if i else 0.0)
            dbe_c[i] += db[i] * m[i]
            dm[i] += be[i] * db[i]
            if i:
                db[i - 1] += al[i] * db[i]
            # a_i = alpha_i a_{i-1};  m_i = mu_i m_{i-1}
            dal_c[i] += da[i] * (a[i - 1] if i else 1.0)
            dmu_c[i] += dm[i] * (m[i - 1] if i else 1.0)
            if i:
                da[i - 1] += al[i] * da[i]
                dm[i - 1] += mm[i] * dm[i]
        dal[sl], dbe[sl], dmu[sl] = dal_c, dbe_c, dmu_c
        dS, dM = dS_in, dM_in
    return dq, dkk, dv, dal, dbe, dmu, det, dS, dM
