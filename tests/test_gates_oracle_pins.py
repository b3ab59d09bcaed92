"""Pins of the gate-parameterisation oracle (Sec. 3.3, "Stability Aware Gating Parameterization") against what the
paper and the mathematics fix, none of them a restatement of its own formulas."""
import numpy as np
import pytest

from oracle import gates_oracle as go


def _inputs(seed=0, B=2, T=5, H=3):
    rng = np.random.default_rng(seed)
    x = [rng.standard_normal((B, T, H)) * 1.5 for _ in range(4)]
    par = dict(a_alpha=rng.uniform(0.2, 2.0, H), b_alpha=rng.standard_normal(H), a_mu=rng.uniform(0.2, 2.0, H),
               b_mu=rng.standard_normal(H), s=0.8, tau=2.5)
    return x, par


def test_upper_bounds_add_up_to_one_and_ranges():
    """alpha_max + beta_max = 1 (the constraint the parameterisation is built to meet): alpha / decay + beta / sigmoid = 1;
    eta in (0, 2); mu in [e^-1, 1]; alpha <= alpha_max < 1; beta < beta_max."""
    x, par = _inputs(1)
    g = go.forward(*x, **par)
    decay = np.exp(-par["a_alpha"] * np.logaddexp(0, x[0] + par["b_alpha"]))
    sig = 1 / (1 + np.exp(-x[2]))
    assert np.allclose(g["alpha"] / decay + g["beta"] / sig, 1.0, atol=1e-12)
    assert (g["eta"] > 0).all() and (g["eta"] < 2).all()
    assert (g["mu"] >= np.exp(-1.0) - 1e-15).all() and (g["mu"] <= 1).all()
    assert (g["alpha"] > 0).all() and (g["alpha"] < 1).all() and (g["beta"] > 0).all() and (g["beta"] < 1).all()


def test_worked_values():
    """x_eta = 0 gives eta = 1; with s = 1 then theta = pi/4 and alpha_max = beta_max = 1/2.  x_alpha + b = 0 gives
    softplus = ln 2, so alpha = 2^-a / 2; x_beta = 0 gives beta = 1/4; x_mu far below the clamp gives mu = e^-1."""
    one = np.zeros((1, 1, 1))
    g = go.forward(one, one - 50.0, one, one, a_alpha=[3.0], b_alpha=[0.0], a_mu=[1.0], b_mu=[100.0], s=1.0, tau=4.0)
    assert g["eta"][0, 0, 0] == pytest.approx(1.0)
    assert g["alpha"][0, 0, 0] == pytest.approx(2.0 ** -3 / 2)
    assert g["beta"][0, 0, 0] == pytest.approx(0.25)
    assert g["mu"][0, 0, 0] == pytest.approx(np.exp(-1.0))     # f_mu = -softplus(50) = -50 < -1: clamped
    g = go.forward(one, one - 50.0, one, one, a_alpha=[3.0], b_alpha=[0.0], a_mu=[1.0], b_mu=[0.0], s=1.0, tau=4.0)
    assert g["mu"][0, 0, 0] == pytest.approx(np.exp(-np.log1p(np.exp(-50.0))))   # not clamped: ~1


def test_s_to_zero_removes_the_constraint_on_alpha_and_kills_beta():
    """theta -> 0: alpha_max -> 1 (alpha is the plain decay gate of Gated DeltaNet / Mamba2), beta_max -> 0."""
    x, par = _inputs(2)
    par["s"] = 1e-9
    g = go.forward(*x, **par)
    assert np.allclose(g["alpha"], np.exp(-par["a_alpha"] * np.logaddexp(0, x[0] + par["b_alpha"])), rtol=1e-12)
    assert np.abs(g["beta"]).max() < 1e-16


def test_backward_matches_central_finite_differences():
    x, par = _inputs(3)
    rng = np.random.default_rng(7)
    d = [rng.standard_normal(x[0].shape) for _ in range(4)]
    loss = lambda xs, p: sum((go.forward(*xs, **p)[k] * dk).sum() for k, dk in zip(("alpha", "beta", "mu", "eta"), d))
    g = go.backward(*x, par["a_alpha"], par["b_alpha"], par["a_mu"], par["b_mu"], par["s"], par["tau"], *d)
    eps = 1e-6
    for i, name in enumerate(("dx_alpha", "dx_mu", "dx_beta", "dx_eta")):
        for idx in [(0, 0, 0), (1, 3, 2), (0, 4, 1)]:
            xp = [t.copy() for t in x]; xm = [t.copy() for t in x]
            xp[i][idx] += eps; xm[i][idx] -= eps
            fd = (loss(xp, par) - loss(xm, par)) / (2 * eps)
            assert g[name][idx] == pytest.approx(fd, rel=1e-6, abs=1e-9), (name, idx)
    for name, key in (("da_alpha", "a_alpha"), ("db_alpha", "b_alpha"), ("da_mu", "a_mu"), ("db_mu", "b_mu")):
        for h in range(3):
            pp = {k: (np.array(v, dtype=float).copy() if np.ndim(v) else v) for k, v in par.items()}
            pm = {k: (np.array(v, dtype=float).copy() if np.ndim(v) else v) for k, v in par.items()}
            pp[key][h] += eps; pm[key][h] -= eps
            fd = (loss(x, pp) - loss(x, pm)) / (2 * eps)
            assert g[name][h] == pytest.approx(fd, rel=1e-6, abs=1e-9), (name, h)


def test_clamped_momentum_gate_passes_no_gradient():
    x, par = _inputs(4)
    x[1][...] = 30.0                       # f_mu = -a softplus(30 + b) far below -1 for a >= 0.2
    par["b_mu"] = np.zeros(3)
    d = [np.ones_like(x[0])] * 4
    g = go.backward(*x, par["a_alpha"], par["b_alpha"], par["a_mu"], par["b_mu"], par["s"], par["tau"], *d)
    assert np.abs(g["dx_mu"]).max() == 0.0 and np.abs(g["da_mu"]).max() == 0.0
