"""Thin ctypes binding of the MDN C-ABI library (include/mdn.h).

Argument marshalling only: every step of the path runs in the HIP kernels of libmdn_hip.so.
PyTorch supplies device memory and the HIP stream.  There is no CPU fallback: a missing
library or a non-CUDA tensor raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmdn_hip.so")

MDN_DTYPE_BF16, MDN_DTYPE_F32 = 0, 1
MDN_WS_FWD, MDN_WS_BWD, MDN_WS_BWD_STATE_ADJOINTS = 0, 1, 2

EXPORTS = ("mdn_version", "mdn_strerror", "mdn_workspace_bytes", "mdn_saved_states_bytes",
           "mdn_saved_operands_bytes", "mdn_chunk_fwd", "mdn_chunk_fwd_noalloc",
           "mdn_chunk_bwd", "mdn_recurrent_step", "mdn_profile_begin", "mdn_profile_end", "mdn_profile_begin_sampled",
           "mdn_profile_launch_counts", "mdn_set_segments",
           "mdn_gates_fwd", "mdn_gates_bwd", "mdn_frontend_fwd", "mdn_frontend_bwd", "mdn_epilogue_fwd",
           "mdn_epilogue_bwd", "mdn_workspace_bytes_varlen", "mdn_chunk_fwd_varlen", "mdn_chunk_bwd_varlen")

KERNEL_NAMES = ("intra_fwd", "scan_fwd", "intra_bwd", "rebuild", "scan_bwd", "grad", "recurrent")


class MdnShape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("T", ctypes.c_int32), ("H", ctypes.c_int32), ("dk", ctypes.c_int32),
                ("dv", ctypes.c_int32), ("C", ctypes.c_int32), ("dtype", ctypes.c_int32), ("scale", ctypes.c_float)]


class MdnGateParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("T", ctypes.c_int32), ("H", ctypes.c_int32), ("a_alpha", ctypes.c_void_p),
                ("b_alpha", ctypes.c_void_p), ("a_mu", ctypes.c_void_p), ("b_mu", ctypes.c_void_p),
                ("s", ctypes.c_float), ("tau", ctypes.c_float), ("mu_log_min", ctypes.c_float)]


class MdnError(RuntimeError):
    pass


_lib = None


def load_library():
    """dlopen libmdn_hip.so (built by __graft_entry__.build()) and declare the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise MdnError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` first")
    lib = ctypes.CDLL(LIB_PATH)
    vp, sp, fp = ctypes.c_void_p, ctypes.POINTER(MdnShape), ctypes.c_void_p
    lib.mdn_version.restype = ctypes.c_int
    lib.mdn_strerror.restype = ctypes.c_char_p
    lib.mdn_strerror.argtypes = [ctypes.c_int]
    lib.mdn_workspace_bytes.restype = ctypes.c_int
    lib.mdn_workspace_bytes.argtypes = [sp, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
    lib.mdn_saved_states_bytes.restype = ctypes.c_int
    lib.mdn_saved_states_bytes.argtypes = [sp, ctypes.POINTER(ctypes.c_size_t)]
    lib.mdn_saved_operands_bytes.restype = ctypes.c_int
    lib.mdn_saved_operands_bytes.argtypes = [sp, ctypes.POINTER(ctypes.c_size_t)]
    lib.mdn_chunk_fwd.restype = ctypes.c_int
    lib.mdn_chunk_fwd.argtypes = [sp] + [vp] * 3 + [fp] * 6 + [vp, fp, fp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.mdn_chunk_fwd_noalloc.restype = ctypes.c_int
    lib.mdn_chunk_fwd_noalloc.argtypes = [sp] + [vp] * 3 + [fp] * 6 + [vp, fp, fp, vp, vp]
    lib.mdn_chunk_bwd.restype = ctypes.c_int
    lib.mdn_chunk_bwd.argtypes = [sp] + [vp] * 3 + [fp] * 6 + [vp] * 4 + [fp] * 2 + [vp] * 3 + [fp] * 6 + \
        [vp, ctypes.c_size_t, vp]
    lib.mdn_recurrent_step.restype = ctypes.c_int
    lib.mdn_recurrent_step.argtypes = [sp] + [vp] * 3 + [fp] * 4 + [fp, fp, vp, vp]
    lib.mdn_profile_begin.restype = ctypes.c_int
    lib.mdn_profile_begin_sampled.restype = ctypes.c_int
    lib.mdn_profile_begin_sampled.argtypes = [ctypes.c_int]
    lib.mdn_profile_launch_counts.restype = ctypes.c_int
    lib.mdn_profile_launch_counts.argtypes = [ctypes.POINTER(ctypes.c_int), ctypes.c_int]
    lib.mdn_profile_end.restype = ctypes.c_int
    lib.mdn_profile_end.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int), ctypes.c_int]
    lib.mdn_set_segments.restype = ctypes.c_int
    lib.mdn_set_segments.argtypes = [ctypes.c_int]
    gp = ctypes.POINTER(MdnGateParams)
    lib.mdn_gates_fwd.restype = ctypes.c_int
    lib.mdn_gates_fwd.argtypes = [gp] + [fp] * 8 + [vp]
    lib.mdn_gates_bwd.restype = ctypes.c_int
    lib.mdn_gates_bwd.argtypes = [gp] + [fp] * 13 + [vp]
    cf = ctypes.c_float
    ip = ctypes.POINTER(ctypes.c_int32)
    lib.mdn_workspace_bytes_varlen.restype = ctypes.c_int
    lib.mdn_workspace_bytes_varlen.argtypes = [sp, ip, ctypes.c_int32, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
    lib.mdn_chunk_fwd_varlen.restype = ctypes.c_int
    lib.mdn_chunk_fwd_varlen.argtypes = [sp, ip, ctypes.c_int32] + [vp] * 3 + [fp] * 6 + [vp, fp, fp, vp, vp, ctypes.c_size_t, vp]
    lib.mdn_chunk_bwd_varlen.restype = ctypes.c_int
    lib.mdn_chunk_bwd_varlen.argtypes = [sp, ip, ctypes.c_int32] + [vp] * 3 + [fp] * 6 + [vp, vp] + [fp] * 2 + [vp] * 3 + \
        [fp] * 6 + [vp, ctypes.c_size_t, vp]
    lib.mdn_frontend_fwd.restype = ctypes.c_int
    lib.mdn_frontend_fwd.argtypes = [sp, vp, vp, vp, fp, cf, vp, vp, vp, vp]
    lib.mdn_frontend_bwd.restype = ctypes.c_int
    lib.mdn_frontend_bwd.argtypes = [sp, vp, vp, vp, fp, cf] + [vp] * 6 + [fp, vp]
    lib.mdn_epilogue_fwd.restype = ctypes.c_int
    lib.mdn_epilogue_fwd.argtypes = [sp, vp, vp, fp, cf, vp, vp]
    lib.mdn_epilogue_bwd.restype = ctypes.c_int
    lib.mdn_epilogue_bwd.argtypes = [sp, vp, vp, fp, cf, vp, vp, vp, fp, vp]
    _lib = lib
    return lib


def _check(rc: int, what: str):
    if rc != 0:
        raise MdnError(f"{what}: {load_library().mdn_strerror(rc).decode()} (code {rc})")


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise MdnError("MDN tensors must live on the GPU (no CPU path exists)")
    if not t.is_contiguous():
        raise MdnError("MDN tensors must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _expect(name, t, shape, dtype, like, optional=False):
    """Shape, dtype, device and layout of one tensor against what the call's q implies.  The C ABI takes raw pointers
    and trusts them: a tensor of the wrong size would be read or written out of bounds on the device, so every tensor
    is checked here, before anything is launched."""
    if t is None:
        if optional:
            return
        raise MdnError(f"{name} is required")
    if tuple(t.shape) != tuple(shape):
        raise MdnError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    if t.dtype != dtype:
        raise MdnError(f"{name}: expected dtype {dtype}, got {t.dtype}")
    if t.device != like.device:
        raise MdnError(f"{name} is on {t.device}, q on {like.device}: all tensors of a call share one device")
    if not t.is_contiguous():
        raise MdnError(f"{name} must be contiguous")


def _expect_bytes(name, t, nbytes, like, optional=True):
    """An opaque buffer (workspace, kept states / operands): at least nbytes, on q's device, contiguous."""
    if t is None:
        if optional:
            return
        raise MdnError(f"{name} is required")
    have = t.numel() * t.element_size()
    if have < nbytes:
        raise MdnError(f"{name}: {have} bytes, the call needs {nbytes}")
    if t.device != like.device:
        raise MdnError(f"{name} is on {t.device}, q on {like.device}: all tensors of a call share one device")
    if not t.is_contiguous():
        raise MdnError(f"{name} must be contiguous")


def _check_inputs(q, k, v, beta, alpha, mu, eta, S0, M0, states_batch=None):
    """The forward inputs that every chunkwise / recurrent call takes; returns (B, T, H, dk, dv)."""
    if q.dim() != 4 or v.dim() != 4:
        raise MdnError(f"q, v must be [B, T, H, d]; got {tuple(q.shape)}, {tuple(v.shape)}")
    _dtype_code(q)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    f32 = torch.float32
    _expect("k", k, (B, T, H, dk), q.dtype, q)
    _expect("v", v, (B, T, H, dv), q.dtype, q)
    for name, g in (("beta", beta), ("alpha", alpha), ("mu", mu)):
        _expect(name, g, (B, T, H), f32, q)
    _expect("eta", eta, (B, T, H), f32, q, optional=True)
    nb = B if states_batch is None else states_batch
    _expect("S0", S0, (nb, H, dk, dv), f32, q, optional=True)
    _expect("M0", M0, (nb, H, dk, dv), f32, q, optional=True)
    if not q.is_contiguous():
        raise MdnError("q must be contiguous")
    return B, T, H, dk, dv


def _f32(t, name):
    if t is not None and t.dtype != torch.float32:
        raise MdnError(f"{name} must be float32")
    return _ptr(t)


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return MDN_DTYPE_BF16
    if t.dtype == torch.float32:
        return MDN_DTYPE_F32
    raise MdnError("q/k/v must be bfloat16 or float32")


def make_shape(q, v, scale=None, C=64) -> MdnShape:
    B, T, H, dk = q.shape
    return MdnShape(B, T, H, dk, v.shape[-1], C, _dtype_code(q), float(dk ** -0.5 if scale is None else scale))


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def workspace_bytes(shape: MdnShape, which: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().mdn_workspace_bytes(ctypes.byref(shape), which, ctypes.byref(n)), "mdn_workspace_bytes")
    return n.value


def saved_states_bytes(shape: MdnShape) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().mdn_saved_states_bytes(ctypes.byref(shape), ctypes.byref(n)), "mdn_saved_states_bytes")
    return n.value


def saved_operands_bytes(shape: MdnShape) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().mdn_saved_operands_bytes(ctypes.byref(shape), ctypes.byref(n)), "mdn_saved_operands_bytes")
    return n.value


def _workspace(shape, which, workspace, device):
    need = workspace_bytes(shape, which)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    return workspace, workspace.numel() * workspace.element_size()


def mdn_chunk_fwd(q, k, v, beta, alpha, mu, eta=None, S0=None, M0=None, scale=None, save_vt=False,
                  save_states=False, save_operands=False, output_final_state=True, workspace=None, out=None,
                  chunk_size=64):
    """Chunkwise forward.  Returns a dict: o, S, M (final states or None), vt, states, operands (or None)."""
    lib = load_library()
    B, T, H, dk, dv = _check_inputs(q, k, v, beta, alpha, mu, eta, S0, M0)
    shape = make_shape(q, v, scale, chunk_size)
    out = {} if out is None else out
    dev = q.device
    o = out.get("o")
    if o is None:
        o = torch.empty((B, T, H, dv), dtype=q.dtype, device=dev)
    S = M = vt = states = operands = None
    if save_operands:
        operands = out.get("operands")
        if operands is None:
            operands = torch.empty(saved_operands_bytes(shape), dtype=torch.uint8, device=dev)
    if output_final_state:
        S = out.get("S") if out.get("S") is not None else torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev)
        M = out.get("M") if out.get("M") is not None else torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev)
    if save_vt:
        vt = out.get("vt") if out.get("vt") is not None else torch.empty((B, T, H, dv), dtype=q.dtype, device=dev)
    if save_states:
        states = out.get("states")
        if states is None:
            states = torch.empty(saved_states_bytes(shape), dtype=torch.uint8, device=dev)  # opaque to the caller
    f32 = torch.float32
    _expect("out['o']", o, (B, T, H, dv), q.dtype, q)
    _expect("out['S']", S, (B, H, dk, dv), f32, q, optional=True)
    _expect("out['M']", M, (B, H, dk, dv), f32, q, optional=True)
    _expect("out['vt']", vt, (B, T, H, dv), q.dtype, q, optional=True)
    if states is not None:
        _expect_bytes("out['states']", states, saved_states_bytes(shape), q)
    if operands is not None:
        _expect_bytes("out['operands']", operands, saved_operands_bytes(shape), q)
    _expect_bytes("workspace", workspace, workspace_bytes(shape, MDN_WS_FWD), q)
    workspace, wbytes = _workspace(shape, MDN_WS_FWD, workspace, dev)
    rc = lib.mdn_chunk_fwd(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _f32(beta, "beta"), _f32(alpha, "alpha"),
                           _f32(mu, "mu"), _f32(eta, "eta"), _f32(S0, "S0"), _f32(M0, "M0"), _ptr(o), _ptr(S),
                           _ptr(M), _ptr(vt), _ptr(states), _ptr(operands), _ptr(workspace), wbytes, _stream())
    _check(rc, "mdn_chunk_fwd")
    return {"o": o, "S": S, "M": M, "vt": vt, "states": states, "operands": operands, "workspace": workspace}


def mdn_chunk_fwd_noalloc(q, k, v, beta, alpha, mu, out, eta=None, S0=None, M0=None, scale=None, chunk_size=64):
    """mdn_chunk_fwd through the entry point that allocates nothing: `out` holds the caller's o and, optionally, S, M
    and vt tensors (all of them preallocated; this function creates no tensor either).  Returns `out`."""
    lib = load_library()
    B, T, H, dk, dv = _check_inputs(q, k, v, beta, alpha, mu, eta, S0, M0)
    shape = make_shape(q, v, scale, chunk_size)
    f32 = torch.float32
    _expect("out['o']", out.get("o"), (B, T, H, dv), q.dtype, q)
    _expect("out['S']", out.get("S"), (B, H, dk, dv), f32, q, optional=True)
    _expect("out['M']", out.get("M"), (B, H, dk, dv), f32, q, optional=True)
    _expect("out['vt']", out.get("vt"), (B, T, H, dv), q.dtype, q, optional=True)
    rc = lib.mdn_chunk_fwd_noalloc(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _f32(beta, "beta"),
                                   _f32(alpha, "alpha"), _f32(mu, "mu"), _f32(eta, "eta"), _f32(S0, "S0"), _f32(M0, "M0"),
                                   _ptr(out["o"]), _ptr(out.get("S")), _ptr(out.get("M")), _ptr(out.get("vt")), _stream())
    _check(rc, "mdn_chunk_fwd_noalloc")
    return out


def mdn_chunk_bwd(q, k, v, beta, alpha, mu, vt, dO, eta=None, S0=None, M0=None, states=None, operands=None,
                  dS_final=None, dM_final=None, scale=None, want_deta=False, want_dstates=True, workspace=None, out=None,
                  chunk_size=64):
    """Chunkwise backward (chunk_size as in the forward call whose vt, states, operands it takes).  Returns a dict:
    dq, dk, dv, dbeta, dalpha, dmu, deta, dS0, dM0."""
    lib = load_library()
    B, T, H, dk, dv_ = _check_inputs(q, k, v, beta, alpha, mu, eta, S0, M0)
    shape = make_shape(q, v, scale, chunk_size)
    out = {} if out is None else out
    dev = q.device
    _expect("vt", vt, (B, T, H, dv_), q.dtype, q)
    _expect("dO", dO, (B, T, H, dv_), q.dtype, q)
    _expect("dS_final", dS_final, (B, H, dk, dv_), torch.float32, q, optional=True)
    _expect("dM_final", dM_final, (B, H, dk, dv_), torch.float32, q, optional=True)
    if states is not None:
        _expect_bytes("states", states, saved_states_bytes(shape), q)
    if operands is not None:
        _expect_bytes("operands", operands, saved_operands_bytes(shape), q)

    def get(name, shp, dt):
        t = out.get(name)
        if t is None:
            return torch.empty(shp, dtype=dt, device=dev)
        _expect(f"out['{name}']", t, shp, dt, q)
        return t

    dq = get("dq", (B, T, H, dk), q.dtype)
    dk_t = get("dk", (B, T, H, dk), q.dtype)
    dv_t = get("dv", (B, T, H, dv_), q.dtype)
    dbeta = get("dbeta", (B, T, H), torch.float32)
    dalpha = get("dalpha", (B, T, H), torch.float32)
    dmu = get("dmu", (B, T, H), torch.float32)
    deta = get("deta", (B, T, H), torch.float32) if want_deta else None
    dS0 = get("dS0", (B, H, dk, dv_), torch.float32) if want_dstates else None
    dM0 = get("dM0", (B, H, dk, dv_), torch.float32) if want_dstates else None
    which = MDN_WS_BWD if dS_final is None and dM_final is None else MDN_WS_BWD_STATE_ADJOINTS
    _expect_bytes("workspace", workspace, workspace_bytes(shape, which), q)
    workspace, wbytes = _workspace(shape, which, workspace, dev)
    rc = lib.mdn_chunk_bwd(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _f32(beta, "beta"), _f32(alpha, "alpha"),
                           _f32(mu, "mu"), _f32(eta, "eta"), _f32(S0, "S0"), _f32(M0, "M0"), _ptr(vt), _ptr(states),
                           _ptr(operands), _ptr(dO), _f32(dS_final, "dS_final"), _f32(dM_final, "dM_final"), _ptr(dq), _ptr(dk_t),
                           _ptr(dv_t), _f32(dbeta, "dbeta"), _f32(dalpha, "dalpha"), _f32(dmu, "dmu"),
                           _f32(deta, "deta"), _f32(dS0, "dS0"), _f32(dM0, "dM0"), _ptr(workspace), wbytes, _stream())
    _check(rc, "mdn_chunk_bwd")
    return {"dq": dq, "dk": dk_t, "dv": dv_t, "dbeta": dbeta, "dalpha": dalpha, "dmu": dmu, "deta": deta,
            "dS0": dS0, "dM0": dM0, "workspace": workspace}


def mdn_recurrent_step(q, k, v, beta, alpha, mu, S, M, eta=None, scale=None, out=None):
    """Recurrent form over the T tokens given; S, M [B,H,dk,dv] fp32 are updated in place.  Returns o."""
    lib = load_library()
    B, T, H, dk, dv = _check_inputs(q, k, v, beta, alpha, mu, eta, S, M)
    if S is None or M is None:
        raise MdnError("S and M are required (they are advanced in place)")
    shape = make_shape(q, v, scale)
    o = out if out is not None else torch.empty((B, T, H, dv), dtype=q.dtype, device=q.device)
    _expect("out", o, (B, T, H, dv), q.dtype, q)
    rc = lib.mdn_recurrent_step(ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _f32(beta, "beta"),
                                _f32(alpha, "alpha"), _f32(mu, "mu"), _f32(eta, "eta"), _f32(S, "S"), _f32(M, "M"),
                                _ptr(o), _stream())
    _check(rc, "mdn_recurrent_step")
    return o


def set_segments(k):
    """Force the number of sequence segments of mdn_chunk_fwd / mdn_chunk_bwd (0 = automatic); returns the old value."""
    return int(load_library().mdn_set_segments(int(k)))


def profile_begin(period=1):
    """Bracket every period-th launch of the library with an event pair (1 = every launch)."""
    _check(load_library().mdn_profile_begin_sampled(int(period)), "mdn_profile_begin_sampled")


def profile_end(with_launch_counts=False):
    """Per-kernel {name: (total_ms, bracketed launches)} since profile_begin(), with_launch_counts: (total_ms, bracketed
    launches, all launches); synchronises the recorded events."""
    n = len(KERNEL_NAMES)
    ms = (ctypes.c_float * n)()
    cnt = (ctypes.c_int * n)()
    every = (ctypes.c_int * n)()
    _check(load_library().mdn_profile_end(ms, cnt, n), "mdn_profile_end")
    _check(load_library().mdn_profile_launch_counts(every, n), "mdn_profile_launch_counts")
    if with_launch_counts:
        return {KERNEL_NAMES[i]: (float(ms[i]), int(cnt[i]), int(every[i])) for i in range(n)}
    return {KERNEL_NAMES[i]: (float(ms[i]), int(cnt[i])) for i in range(n)}


def _gate_params(x, a_alpha, b_alpha, a_mu, b_mu, s, tau, mu_log_min):
    if x.dim() != 3:
        raise MdnError(f"gate projections must be [B, T, H]; got {tuple(x.shape)}")
    B, T, H = x.shape
    for name, t in (("a_alpha", a_alpha), ("b_alpha", b_alpha), ("a_mu", a_mu), ("b_mu", b_mu)):
        _expect(name, t, (H,), torch.float32, x)
    return MdnGateParams(B, T, H, _f32(a_alpha, "a_alpha").value, _f32(b_alpha, "b_alpha").value,
                         _f32(a_mu, "a_mu").value, _f32(b_mu, "b_mu").value, float(s), float(tau), float(mu_log_min))


def mdn_gates_fwd(x_alpha, x_mu, x_beta, x_eta, a_alpha, b_alpha, a_mu, b_mu, s, tau, mu_log_min=-1.0):
    """Gate parameterisation: projections [B,T,H] fp32 -> dict(alpha, beta, mu, eta), each [B,T,H] fp32."""
    lib = load_library()
    for name, t in (("x_alpha", x_alpha), ("x_mu", x_mu), ("x_beta", x_beta), ("x_eta", x_eta)):
        _expect(name, t, x_alpha.shape, torch.float32, x_alpha)
    p = _gate_params(x_alpha, a_alpha, b_alpha, a_mu, b_mu, s, tau, mu_log_min)
    out = {k: torch.empty_like(x_alpha) for k in ("alpha", "beta", "mu", "eta")}
    rc = lib.mdn_gates_fwd(ctypes.byref(p), _f32(x_alpha, "x_alpha"), _f32(x_mu, "x_mu"), _f32(x_beta, "x_beta"),
                           _f32(x_eta, "x_eta"), _ptr(out["alpha"]), _ptr(out["beta"]), _ptr(out["mu"]), _ptr(out["eta"]),
                           _stream())
    _check(rc, "mdn_gates_fwd")
    return out


def mdn_gates_bwd(x_alpha, x_mu, x_beta, x_eta, a_alpha, b_alpha, a_mu, b_mu, s, tau, dalpha, dbeta, dmu, deta,
                  mu_log_min=-1.0, want_dparams=True):
    """Adjoint of mdn_gates_fwd: dict(dx_alpha, dx_mu, dx_beta, dx_eta [B,T,H]; dparams [4,H] = da_alpha, db_alpha,
    da_mu, db_mu, or None)."""
    lib = load_library()
    for name, t in (("x_alpha", x_alpha), ("x_mu", x_mu), ("x_beta", x_beta), ("x_eta", x_eta), ("dalpha", dalpha),
                    ("dbeta", dbeta), ("dmu", dmu), ("deta", deta)):
        _expect(name, t, x_alpha.shape, torch.float32, x_alpha)
    p = _gate_params(x_alpha, a_alpha, b_alpha, a_mu, b_mu, s, tau, mu_log_min)
    out = {k: torch.empty_like(x_alpha) for k in ("dx_alpha", "dx_mu", "dx_beta", "dx_eta")}
    out["dparams"] = torch.empty((4, x_alpha.shape[2]), dtype=torch.float32, device=x_alpha.device) if want_dparams else None
    rc = lib.mdn_gates_bwd(ctypes.byref(p), _f32(x_alpha, "x_alpha"), _f32(x_mu, "x_mu"), _f32(x_beta, "x_beta"),
                           _f32(x_eta, "x_eta"), _f32(dalpha, "dalpha"), _f32(dbeta, "dbeta"), _f32(dmu, "dmu"),
                           _f32(deta, "deta"), _ptr(out["dx_alpha"]), _ptr(out["dx_mu"]), _ptr(out["dx_beta"]),
                           _ptr(out["dx_eta"]), _ptr(out["dparams"]), _stream())
    _check(rc, "mdn_gates_bwd")
    return out


def _check_frontend(x_q, x_k, x_v, d):
    if x_q.dim() != 4 or x_v.dim() != 4:
        raise MdnError(f"x_q, x_v must be [B, T, H, d]; got {tuple(x_q.shape)}, {tuple(x_v.shape)}")
    _dtype_code(x_q)
    B, T, H, dk = x_q.shape
    _expect("x_q", x_q, (B, T, H, dk), x_q.dtype, x_q)
    _expect("x_k", x_k, (B, T, H, dk), x_q.dtype, x_q)
    _expect("x_v", x_v, (B, T, H, x_v.shape[-1]), x_q.dtype, x_q)
    _expect("d", d, (H,), torch.float32, x_q)


def _check_epilogue(o, g, w, dy=None):
    if o.dim() != 4:
        raise MdnError(f"o must be [B, T, H, dv]; got {tuple(o.shape)}")
    _dtype_code(o)
    _expect("o", o, o.shape, o.dtype, o)
    _expect("g", g, o.shape, o.dtype, o)
    _expect("w", w, (o.shape[-1],), torch.float32, o)
    _expect("dy", dy, o.shape, o.dtype, o, optional=True)


def mdn_frontend_fwd(x_q, x_k, x_v, d, eps=1e-6):
    """SiLU, output correction and L2 norms on the short-convolution outputs -> dict(q, k, v)."""
    _check_frontend(x_q, x_k, x_v, d)
    shape = make_shape(x_q, x_v, 1.0)
    out = {"q": torch.empty_like(x_q), "k": torch.empty_like(x_k), "v": torch.empty_like(x_v)}
    rc = load_library().mdn_frontend_fwd(ctypes.byref(shape), _ptr(x_q), _ptr(x_k), _ptr(x_v), _f32(d, "d"), float(eps),
                                         _ptr(out["q"]), _ptr(out["k"]), _ptr(out["v"]), _stream())
    _check(rc, "mdn_frontend_fwd")
    return out


def mdn_frontend_bwd(x_q, x_k, x_v, d, dq, dk, dv, eps=1e-6, want_dd=True):
    _check_frontend(x_q, x_k, x_v, d)
    _expect("dq", dq, x_q.shape, x_q.dtype, x_q)
    _expect("dk", dk, x_k.shape, x_q.dtype, x_q)
    _expect("dv", dv, x_v.shape, x_q.dtype, x_q)
    shape = make_shape(x_q, x_v, 1.0)
    out = {"dx_q": torch.empty_like(x_q), "dx_k": torch.empty_like(x_k), "dx_v": torch.empty_like(x_v),
           "dd": torch.empty_like(d) if want_dd else None}
    rc = load_library().mdn_frontend_bwd(ctypes.byref(shape), _ptr(x_q), _ptr(x_k), _ptr(x_v), _f32(d, "d"), float(eps),
                                         _ptr(dq), _ptr(dk), _ptr(dv), _ptr(out["dx_q"]), _ptr(out["dx_k"]),
                                         _ptr(out["dx_v"]), _ptr(out["dd"]), _stream())
    _check(rc, "mdn_frontend_bwd")
    return out


def mdn_epilogue_fwd(o, g, w, eps=1e-6):
    """Head-wise RMS norm with weight w [dv] times sigmoid(g) -> y."""
    _check_epilogue(o, g, w)
    B, T, H, dv = o.shape
    shape = MdnShape(B, T, H, dv, dv, 64, _dtype_code(o), 1.0)
    y = torch.empty_like(o)
    rc = load_library().mdn_epilogue_fwd(ctypes.byref(shape), _ptr(o), _ptr(g), _f32(w, "w"), float(eps), _ptr(y), _stream())
    _check(rc, "mdn_epilogue_fwd")
    return y


def mdn_epilogue_bwd(o, g, w, dy, eps=1e-6, want_dw=True):
    _check_epilogue(o, g, w, dy)
    B, T, H, dv = o.shape
    shape = MdnShape(B, T, H, dv, dv, 64, _dtype_code(o), 1.0)
    out = {"do": torch.empty_like(o), "dg": torch.empty_like(g), "dw": torch.empty_like(w) if want_dw else None}
    rc = load_library().mdn_epilogue_bwd(ctypes.byref(shape), _ptr(o), _ptr(g), _f32(w, "w"), float(eps), _ptr(dy),
                                         _ptr(out["do"]), _ptr(out["dg"]), _ptr(out["dw"]), _stream())
    _check(rc, "mdn_epilogue_bwd")
    return out


def _cu(cu_seqlens, T):
    cu = [int(x) for x in cu_seqlens]
    if len(cu) < 2 or cu[0] != 0 or cu[-1] != T or any(b <= a for a, b in zip(cu, cu[1:])):
        raise MdnError(f"cu_seqlens must rise from 0 to T = {T} without empty sequences; got {cu[:8]}{'...' if len(cu) > 8 else ''}")
    return (ctypes.c_int32 * len(cu))(*cu), len(cu) - 1


def _varlen_workspace(shape, cu, n, which, device):
    need = ctypes.c_size_t(0)
    _check(load_library().mdn_workspace_bytes_varlen(ctypes.byref(shape), cu, n, which, ctypes.byref(need)),
           "mdn_workspace_bytes_varlen")
    return torch.empty(max(need.value, 16), dtype=torch.uint8, device=device), need.value


def mdn_chunk_fwd_varlen(q, k, v, beta, alpha, mu, cu_seqlens, eta=None, S0=None, M0=None, scale=None, save_vt=False,
                         want_states=True):
    """Packed variable-length forward: q, k, v [1, T, H, d], gates [1, T, H], cu_seqlens a host sequence of n + 1
    offsets; states [n, H, dk, dv].  Returns dict(o, S, M, vt); S, M are None with want_states=False (without initial
    states either, the library then runs the batch as one stream of tokens)."""
    if q.dim() != 4 or q.shape[0] != 1:
        raise MdnError(f"packed batches are [1, T, H, d]; got q {tuple(q.shape)}")
    cu, n = _cu(cu_seqlens, q.shape[1])
    _, T, H, dk, dv = _check_inputs(q, k, v, beta, alpha, mu, eta, S0, M0, states_batch=n)
    shape = make_shape(q, v, scale)
    o = torch.empty_like(v)
    S = torch.empty((n, H, dk, dv), dtype=torch.float32, device=q.device) if want_states else None
    M = torch.empty_like(S) if want_states else None
    vt = torch.empty_like(v) if save_vt else None
    ws, nb = _varlen_workspace(shape, cu, n, MDN_WS_FWD, q.device)
    rc = load_library().mdn_chunk_fwd_varlen(ctypes.byref(shape), cu, n, _ptr(q), _ptr(k), _ptr(v), _f32(beta, "beta"),
                                             _f32(alpha, "alpha"), _f32(mu, "mu"), _f32(eta, "eta"), _f32(S0, "S0"),
                                             _f32(M0, "M0"), _ptr(o), _ptr(S), _ptr(M), _ptr(vt), _ptr(ws), nb, _stream())
    _check(rc, "mdn_chunk_fwd_varlen")
    return {"o": o, "S": S, "M": M, "vt": vt}


def mdn_chunk_bwd_varlen(q, k, v, beta, alpha, mu, vt, dO, cu_seqlens, eta=None, S0=None, M0=None, dS_final=None,
                         dM_final=None, scale=None, want_deta=False, want_state_grads=True):
    """Packed variable-length backward.  Returns dict(dq, dk, dv, dbeta, dalpha, dmu, deta, dS0, dM0); dS0, dM0 are
    None with want_state_grads=False (with no initial states and no adjoints of the final states either, the
    library then runs the batch as one stream of tokens)."""
    if q.dim() != 4 or q.shape[0] != 1:
        raise MdnError(f"packed batches are [1, T, H, d]; got q {tuple(q.shape)}")
    cu, n = _cu(cu_seqlens, q.shape[1])
    _, T, H, dk, dv_ = _check_inputs(q, k, v, beta, alpha, mu, eta, S0, M0, states_batch=n)
    _expect("vt", vt, (1, T, H, dv_), q.dtype, q)
    _expect("dO", dO, (1, T, H, dv_), q.dtype, q)
    _expect("dS_final", dS_final, (n, H, dk, dv_), torch.float32, q, optional=True)
    _expect("dM_final", dM_final, (n, H, dk, dv_), torch.float32, q, optional=True)
    shape = make_shape(q, v, scale)
    out = {"dq": torch.empty_like(q), "dk": torch.empty_like(k), "dv": torch.empty_like(v)}
    for name in ("dbeta", "dalpha", "dmu"):
        out[name] = torch.empty_like(beta)
    out["deta"] = torch.empty_like(beta) if want_deta else None
    out["dS0"] = torch.empty((n, H, dk, dv_), dtype=torch.float32, device=q.device) if want_state_grads else None
    out["dM0"] = torch.empty_like(out["dS0"]) if want_state_grads else None
    ws, nb = _varlen_workspace(shape, cu, n, MDN_WS_BWD, q.device)
    rc = load_library().mdn_chunk_bwd_varlen(ctypes.byref(shape), cu, n, _ptr(q), _ptr(k), _ptr(v), _f32(beta, "beta"),
                                             _f32(alpha, "alpha"), _f32(mu, "mu"), _f32(eta, "eta"), _f32(S0, "S0"),
                                             _f32(M0, "M0"), _ptr(vt), _ptr(dO), _f32(dS_final, "dS_final"),
                                             _f32(dM_final, "dM_final"), _ptr(out["dq"]), _ptr(out["dk"]), _ptr(out["dv"]),
                                             _ptr(out["dbeta"]), _ptr(out["dalpha"]), _ptr(out["dmu"]), _ptr(out["deta"]),
                                             _ptr(out["dS0"]), _ptr(out["dM0"]), _ptr(ws), nb, _stream())
    _check(rc, "mdn_chunk_bwd_varlen")
    return out
