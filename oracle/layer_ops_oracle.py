"""fp64 numpy oracle of the elementwise operations around the momentum delta rule in the MDN layer (Sec. 3.3,
architecture paragraph) -- TEST INFRASTRUCTURE ONLY (tests and smoke checks may import it; the product never does).

Front end, per token and head (x_q, x_k, x_v are the short-convolution outputs, [B, T, H, d]):
    q' = SiLU(x_q),  k' = SiLU(x_k),  v = SiLU(x_v),     SiLU(x) = x sigmoid(x)
    q  = L2Norm(q' - d_h k')          (the output correction, applied before the normalisation)
    k  = L2Norm(k')                   L2Norm(x) = x / sqrt(sum x^2 + eps)
Back end (before the output projection), per token and head:
    y = sigmoid(g) * RMSNorm(o),      RMSNorm(o) = w * o / sqrt(mean(o^2) + eps)      (w: [dv], shared by the heads)

Each `*_forward` is the definition written out; each `*_backward` its adjoint, derivative by derivative.
"""
from __future__ import annotations

import numpy as np


def _sig(x):
    return 1.0 / (1.0 + np.exp(-x))


def _f64(*a):
    return [np.asarray(t, dtype=np.float64) for t in a]


def frontend_forward(x_q, x_k, x_v, d, eps=1e-6):
    """x_q, x_k [B,T,H,dk], x_v [B,T,H,dv], d [H] -> dict(q, k, v)."""
    xq, xk, xv, d = _f64(x_q, x_k, x_v, d)
    qs, ks = xq * _sig(xq), xk * _sig(xk)
    qc = qs - d[None, None, :, None] * ks
    q = qc / np.sqrt((qc * qc).sum(-1, keepdims=True) + eps)
    k = ks / np.sqrt((ks * ks).sum(-1, keepdims=True) + eps)
    return {"q": q, "k": k, "v": xv * _sig(xv)}


def _dsilu(x):
    s = _sig(x)
    return s * (1.0 + x * (1.0 - s))


def _l2norm_bwd(x, dy, eps):
    """y = x / sqrt(sum x^2 + eps):  dx = (dy - y <y, dy>) / sqrt(sum x^2 + eps)."""
    r = np.sqrt((x * x).sum(-1, keepdims=True) + eps)
    y = x / r
    return (dy - y * (y * dy).sum(-1, keepdims=True)) / r


def frontend_backward(x_q, x_k, x_v, d, dq, dk, dv, eps=1e-6):
    """Adjoint of frontend_forward -> dict(dx_q, dx_k, dx_v, dd [H])."""
    xq, xk, xv, d, dq, dk, dv = _f64(x_q, x_k, x_v, d, dq, dk, dv)
    dh = d[None, None, :, None]
    qs, ks = xq * _sig(xq), xk * _sig(xk)
    dqc = _l2norm_bwd(qs - dh * ks, dq, eps)
    dks = _l2norm_bwd(ks, dk, eps) - dh * dqc
    return {"dx_q": dqc * _dsilu(xq), "dx_k": dks * _dsilu(xk), "dx_v": dv * _dsilu(xv),
            "dd": -(dqc * ks).sum(axis=(0, 1, 3))}


def epilogue_forward(o, g, w, eps=1e-6):
    """o, g [B,T,H,dv], w [dv] -> y [B,T,H,dv]."""
    o, g, w = _f64(o, g, w)
    return _sig(g) * w * o / np.sqrt((o * o).mean(-1, keepdims=True) + eps)


def epilogue_backward(o, g, w, dy, eps=1e-6):
    """Adjoint of epilogue_forward -> dict(do, dg, dw [dv])."""
    o, g, w, dy = _f64(o, g, w, dy)
    r = np.sqrt((o * o).mean(-1, keepdims=True) + eps)
    n = o / r
    sg = _sig(g)
    dn = dy * sg * w                                        # adjoint of the normalised vector
    do = (dn - n * (n * dn).mean(-1, keepdims=True)) / r
    return {"do": do, "dg": dy * w * n * sg * (1.0 - sg), "dw": (dy * sg * n).sum(axis=(0, 1, 2))}
