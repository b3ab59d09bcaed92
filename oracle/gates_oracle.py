"""fp64 numpy oracle of the stability-aware gate parameterisation (Sec. 3.3, "Stability Aware Gating
Parameterization") -- TEST INFRASTRUCTURE ONLY (tests and smoke checks may import it; the product never does).

From the per-head projections x_alpha, x_mu, x_beta, x_eta of a token (each [B, T, H]) to the linear-domain gates
that the momentum delta rule takes:

    eta   = tanh(x_eta / tau) + 1                                   in (0, 2)
    theta = arctan(eta * s),  alpha_max = cos^2 theta,  beta_max = sin^2 theta      (alpha_max + beta_max = 1)
    alpha = exp(f_alpha(x_alpha) + log alpha_max),   f(x) = -a * softplus(x + b)    (a > 0, b per head)
    mu    = exp(max(f_mu(x_mu), mu_log_min))                        (the clamp keeps the momentum from vanishing)
    beta  = sigmoid(x_beta) * beta_max

`forward` is that definition written out; `backward` is its adjoint, derivative by derivative.
"""
from __future__ import annotations

import numpy as np


def _softplus(x):
    return np.logaddexp(0.0, x)


def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def forward(x_alpha, x_mu, x_beta, x_eta, a_alpha, b_alpha, a_mu, b_mu, s, tau, mu_log_min=-1.0):
    """All x_* are [B, T, H]; a_*, b_* are [H].  Returns dict(alpha, beta, mu, eta), each [B, T, H] float64."""
    xa, xm, xb, xe = (np.asarray(t, dtype=np.float64) for t in (x_alpha, x_mu, x_beta, x_eta))
    aa, ba, am, bm = (np.asarray(t, dtype=np.float64) for t in (a_alpha, b_alpha, a_mu, b_mu))
    eta = np.tanh(xe / tau) + 1.0
    theta = np.arctan(eta * s)
    alpha_max = np.cos(theta) ** 2
    beta_max = np.sin(theta) ** 2
    alpha = np.exp(-aa * _softplus(xa + ba) + np.log(alpha_max))
    mu = np.exp(np.maximum(-am * _softplus(xm + bm), mu_log_min))
    beta = _sigmoid(xb) * beta_max
    return {"alpha": alpha, "beta": beta, "mu": mu, "eta": eta}


def backward(x_alpha, x_mu, x_beta, x_eta, a_alpha, b_alpha, a_mu, b_mu, s, tau, d_alpha, d_beta, d_mu, d_eta,
             mu_log_min=-1.0):
    """Adjoint of `forward` for L = <alpha, d_alpha> + <beta, d_beta> + <mu, d_mu> + <eta, d_eta>.
    Returns dict(dx_alpha, dx_mu, dx_beta, dx_eta [B,T,H]; da_alpha, db_alpha, da_mu, db_mu [H])."""
    xa, xm, xb, xe = (np.asarray(t, dtype=np.float64) for t in (x_alpha, x_mu, x_beta, x_eta))
    aa, ba, am, bm = (np.asarray(t, dtype=np.float64) for t in (a_alpha, b_alpha, a_mu, b_mu))
    da, db, dm, de = (np.asarray(t, dtype=np.float64) for t in (d_alpha, d_beta, d_mu, d_eta))
    th = np.tanh(xe / tau)
    eta = th + 1.0
    u = eta * s
    den = 1.0 + u * u                      # alpha_max = 1 / den, beta_max = u^2 / den
    alpha_max, beta_max = 1.0 / den, u * u / den
    dmax_deta = 2.0 * u * s / den ** 2     # d beta_max / d eta = - d alpha_max / d eta
    decay = np.exp(-aa * _softplus(xa + ba))
    alpha = alpha_max * decay
    sig_b = _sigmoid(xb)
    g = -am * _softplus(xm + bm)
    live = g > mu_log_min                  # the clamp passes no gradient
    mu = np.exp(np.maximum(g, mu_log_min))
    # d alpha / d f_alpha = alpha;  d f / d x = -a sigmoid(x + b),  d f / d a = -softplus(x + b),  d f / d b = d f / d x
    dfa = da * alpha
    dx_alpha = dfa * (-aa * _sigmoid(xa + ba))
    dfm = np.where(live, dm * mu, 0.0)
    dx_mu = dfm * (-am * _sigmoid(xm + bm))
    dx_beta = db * beta_max * sig_b * (1.0 - sig_b)
    deta_total = de + da * decay * (-dmax_deta) + db * sig_b * dmax_deta
    dx_eta = deta_total * (1.0 - th * th) / tau
    red = lambda t: t.sum(axis=(0, 1))
    return {"dx_alpha": dx_alpha, "dx_mu": dx_mu, "dx_beta": dx_beta, "dx_eta": dx_eta,
            "da_alpha": red(dfa * (-_softplus(xa + ba))), "db_alpha": red(dx_alpha),
            "da_mu": red(dfm * (-_softplus(xm + bm))), "db_mu": red(dx_mu)}
