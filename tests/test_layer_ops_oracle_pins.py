"""Pins of the oracle of the layer's elementwise front and back end (Sec. 3.3) against invariants and limits that do
not restate its formulas."""
import numpy as np
import pytest

from oracle import layer_ops_oracle as lo


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def test_frontend_unit_norms_silu_values_and_zero_correction():
    xq, xk, xv = _rand(1, 2, 5, 3, 8), _rand(2, 2, 5, 3, 8), _rand(3, 2, 5, 3, 6)
    d = np.array([0.0, 0.3, -0.5])
    f = lo.frontend_forward(xq, xk, xv, d, eps=0.0)
    assert np.allclose(np.linalg.norm(f["q"], axis=-1), 1.0) and np.allclose(np.linalg.norm(f["k"], axis=-1), 1.0)
    # SiLU at known points: 0 -> 0, large x -> x, 1 -> 1 / (1 + e^-1)
    v = lo.frontend_forward(xq, xk, np.array([0.0, 40.0, 1.0]).reshape(1, 1, 1, 3).repeat(3, 2), d[:3])["v"][0, 0, 0]
    assert v[0] == 0.0 and v[1] == pytest.approx(40.0) and v[2] == pytest.approx(1.0 / (1.0 + np.exp(-1.0)))
    # head 0 has d = 0: q is the normalised SiLU(x_q), whatever k is
    f2 = lo.frontend_forward(xq, _rand(9, 2, 5, 3, 8), xv, d, eps=0.0)
    assert np.allclose(f["q"][:, :, 0], f2["q"][:, :, 0])
    assert not np.allclose(f["q"][:, :, 1], f2["q"][:, :, 1])
    # the correction is applied BEFORE the normalisation: q is parallel to SiLU(x_q) - d SiLU(x_k)
    silu = lambda x: x / (1 + np.exp(-x))
    c = silu(xq) - d[None, None, :, None] * silu(xk)
    cos = (c * f["q"]).sum(-1) / np.linalg.norm(c, axis=-1)
    assert np.allclose(cos, 1.0)


def test_epilogue_scale_invariance_and_limits():
    o, g, w = _rand(4, 2, 4, 3, 8), _rand(5, 2, 4, 3, 8), _rand(6, 8)
    y = lo.epilogue_forward(o, g, w, eps=0.0)
    assert np.allclose(lo.epilogue_forward(3.7 * o, g, w, eps=0.0), y)             # RMSNorm ignores the scale of o
    big = lo.epilogue_forward(o, np.full_like(g, 50.0), np.ones(8), eps=0.0)       # open gate, unit weight
    assert np.allclose((big ** 2).mean(-1), 1.0)                                   # unit root-mean-square
    assert np.allclose(lo.epilogue_forward(o, np.zeros_like(g), w, eps=0.0), 0.5 * lo.epilogue_forward(o, np.full_like(g, 50.0), w, eps=0.0))
    const = lo.epilogue_forward(np.full((1, 1, 1, 8), -2.0), np.full((1, 1, 1, 8), 50.0), np.arange(8.0), eps=0.0)
    assert np.allclose(const[0, 0, 0], -np.arange(8.0))                            # a constant vector normalises to its sign


@pytest.mark.parametrize("eps", [1e-6, 1e-2])
def test_backwards_match_central_finite_differences(eps):
    xq, xk, xv = _rand(11, 1, 3, 2, 6), _rand(12, 1, 3, 2, 6), _rand(13, 1, 3, 2, 5)
    d = np.array([0.2, -0.4])
    dq, dk, dv = _rand(14, 1, 3, 2, 6), _rand(15, 1, 3, 2, 6), _rand(16, 1, 3, 2, 5)
    loss = lambda a, b, c, dd: sum((lo.frontend_forward(a, b, c, dd, eps)[n] * t).sum() for n, t in (("q", dq), ("k", dk), ("v", dv)))
    g = lo.frontend_backward(xq, xk, xv, d, dq, dk, dv, eps)
    h = 1e-6
    for name, arr, pos in (("dx_q", xq, 0), ("dx_k", xk, 1), ("dx_v", xv, 2)):
        for idx in [(0, 0, 0, 0), (0, 2, 1, 3), (0, 1, 0, 4)]:
            args_p = [xq.copy(), xk.copy(), xv.copy()]; args_m = [xq.copy(), xk.copy(), xv.copy()]
            args_p[pos][idx] += h; args_m[pos][idx] -= h
            fd = (loss(*args_p, d) - loss(*args_m, d)) / (2 * h)
            assert g[name][idx] == pytest.approx(fd, rel=1e-6, abs=1e-9), (name, idx)
    for hh in range(2):
        dp, dm = d.copy(), d.copy(); dp[hh] += h; dm[hh] -= h
        assert g["dd"][hh] == pytest.approx((loss(xq, xk, xv, dp) - loss(xq, xk, xv, dm)) / (2 * h), rel=1e-6, abs=1e-9)
    o, gg, w, dy = _rand(17, 1, 3, 2, 5), _rand(18, 1, 3, 2, 5), _rand(19, 5), _rand(20, 1, 3, 2, 5)
    eloss = lambda a, b, c: (lo.epilogue_forward(a, b, c, eps) * dy).sum()
    e = lo.epilogue_backward(o, gg, w, dy, eps)
    for name, pos in (("do", 0), ("dg", 1)):
        for idx in [(0, 0, 0, 0), (0, 2, 1, 3)]:
            ap = [o.copy(), gg.copy()]; am = [o.copy(), gg.copy()]
            ap[pos][idx] += h; am[pos][idx] -= h
            assert e[name][idx] == pytest.approx((eloss(*ap, w) - eloss(*am, w)) / (2 * h), rel=1e-6, abs=1e-9), (name, idx)
    for j in range(5):
        wp, wm = w.copy(), w.copy(); wp[j] += h; wm[j] -= h
        assert e["dw"][j] == pytest.approx((eloss(o, gg, wp) - eloss(o, gg, wm)) / (2 * h), rel=1e-6, abs=1e-9)
