"""ctypes front end of the fp64 C oracle (oracle/mdn_oracle.c) -- TEST INFRASTRUCTURE ONLY.

The arithmetic lives in the C file: the token-by-token recurrence of Sec. 3.1
(Eq. Mt.recurrent / St.recurrent, with p = alpha*k and the correction value v~) in the
operation order of the recurrent form in Appendix E, and its hand-derived token-level
adjoint.  This module only marshals numpy arrays; it holds none of the method's arithmetic.

Only tests, `__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py` may import it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mdn_oracle.c")
_LIB = os.path.join(_HERE, "libmdn_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over the independent (batch, head) pairs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        i = ctypes.c_int
        lib.mdn_oracle_forward.restype = i
        lib.mdn_oracle_forward.argtypes = [i, i, i, i, i, ctypes.c_double] + [dp] * 13 + [i]
        lib.mdn_oracle_backward.restype = i
        lib.mdn_oracle_backward.argtypes = [i, i, i, i, i, ctypes.c_double] + [dp] * 21 + [i]
        _lib = lib
    return _lib


def _in(a, shape=None):
    if a is None:
        return None, None
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _out(shape):
    a = np.zeros(shape, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def forward(q, k, v, alpha, beta, mu, eta=None, S0=None, M0=None, scale=None, nthreads=0):
    """o, S_T, M_T, v~ = MDN(q, k, v, alpha, beta, mu, eta) token by token in fp64.

    q, k: [B,T,H,dk]; v: [B,T,H,dv]; gates: [B,T,H]; states: [B,H,dk,dv].
    Returns a dict with o [B,T,H,dv], S, M [B,H,dk,dv], vt [B,T,H,dv] and `threads`.
    """
    lib = _load()
    q = np.asarray(q)
    B, T, H, dk = q.shape
    dv = np.asarray(v).shape[-1]
    if scale is None:
        scale = dk ** -0.5
    qa, qp = _in(q)
    ka, kp = _in(k, (B, T, H, dk))
    va, vp = _in(v, (B, T, H, dv))
    aa, ap = _in(alpha, (B, T, H))
    ba, bp = _in(beta, (B, T, H))
    ma, mp = _in(mu, (B, T, H))
    ea, ep = _in(eta, (B, T, H))
    s0, s0p = _in(S0, (B, H, dk, dv))
    m0, m0p = _in(M0, (B, H, dk, dv))
    o, op = _out((B, T, H, dv))
    S, Sp = _out((B, H, dk, dv))
    M, Mp = _out((B, H, dk, dv))
    vt, vtp = _out((B, T, H, dv))
    r = lib.mdn_oracle_forward(B, T, H, dk, dv, float(scale), qp, kp, vp, ap, bp, mp, ep, s0p, m0p,
                               op, Sp, Mp, vtp, int(nthreads))
    if r < 0:
        raise MemoryError("mdn_oracle_forward: allocation failed")
    return {"o": o, "S": S, "M": M, "vt": vt, "threads": r}


def backward(q, k, v, alpha, beta, mu, dO, eta=None, S0=None, M0=None, dS_T=None, dM_T=None, scale=None,
             nthreads=0):
    """Gradients of sum(o*dO) + <S_T,dS_T> + <M_T,dM_T> w.r.t. every input, in fp64.

    Returns a dict with dq, dk, dv, dalpha, dbeta, dmu, deta, dS0, dM0 and `threads`.
    deta is the gradient w.r.t. eta also when eta was omitted (evaluated at eta = 1).
    """
    lib = _load()
    q = np.asarray(q)
    B, T, H, dk = q.shape
    dv = np.asarray(v).shape[-1]
    if scale is None:
        scale = dk ** -0.5
    qa, qp = _in(q)
    ka, kp = _in(k, (B, T, H, dk))
    va, vp = _in(v, (B, T, H, dv))
    aa, ap = _in(alpha, (B, T, H))
    ba, bp = _in(beta, (B, T, H))
    ma, mp = _in(mu, (B, T, H))
    ea, ep = _in(eta, (B, T, H))
    s0, s0p = _in(S0, (B, H, dk, dv))
    m0, m0p = _in(M0, (B, H, dk, dv))
    do, dop = _in(dO, (B, T, H, dv))
    dst, dstp = _in(dS_T, (B, H, dk, dv))
    dmt, dmtp = _in(dM_T, (B, H, dk, dv))
    dq, dqp = _out((B, T, H, dk))
    dk_, dkp = _out((B, T, H, dk))
    dv_, dvp = _out((B, T, H, dv))
    da, dap = _out((B, T, H))
    db, dbp = _out((B, T, H))
    dm, dmp = _out((B, T, H))
    de, dep = _out((B, T, H))
    ds0, ds0p = _out((B, H, dk, dv))
    dm0, dm0p = _out((B, H, dk, dv))
    r = lib.mdn_oracle_backward(B, T, H, dk, dv, float(scale), qp, kp, vp, ap, bp, mp, ep, s0p, m0p, dop,
                                dstp, dmtp, dqp, dkp, dvp, dap, dbp, dmp, dep, ds0p, dm0p, int(nthreads))
    if r < 0:
        raise MemoryError("mdn_oracle_backward: allocation failed")
    return {"dq": dq, "dk": dk_, "dv": dv_, "dalpha": da, "dbeta": db, "dmu": dm, "deta": de,
            "dS0": ds0, "dM0": dm0, "threads": r}
