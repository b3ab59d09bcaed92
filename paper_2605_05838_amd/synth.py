"""Seeded synthetic inputs for the Momentum DeltaNet hot path.

This module only draws random numbers and rounds them; it holds none of the method's
arithmetic, so both the GPU path's callers and the CPU oracle's tests may use it.

The tensors stand in for the activations of the paper's 400M / 1.3B layers (Sec. 4.2),
which need trained weights: shapes follow those model scales, value distributions follow
Sec. 3.3 (L2-normalised q and k, sigmoid step size beta, decay alpha = exp(-softplus(.)) =
sigmoid(logit), momentum gate mu clamped from below at log(mu) = -1, eta = 1).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

LOG_MU_MIN = -1.0  # default clamp of log(mu), Sec. 3.3


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values that are already bfloat16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16).reshape(x.shape)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(b.shape)


def _sigmoid(z):
    z = z.astype(np.float64)
    return 1.0 / (1.0 + np.exp(-z))


@dataclass
class Workload:
    name: str
    B: int
    T: int
    H: int
    dk: int
    dv: int
    C: int
    dtype: str  # "bf16" | "f32": storage type of q, k, v, o, dO and their gradients
    backward: bool
    seed: int
    alpha_logit_mean: float = 0.0
    mu_logit_mean: float = 0.0
    s0_std: float = 0.0
    with_eta: bool = False
    log_mu_min: float = LOG_MU_MIN
    arrays: dict = field(default_factory=dict, repr=False)

    @property
    def scale(self) -> float:
        return float(self.dk) ** -0.5

    @property
    def tokens(self) -> int:
        return self.B * self.T


# The five measurement configurations (shapes, dtypes, gate biases, seeds).
CONFIGS = {
    0: dict(name="c0_tiny_f32_fwd", B=1, T=256, H=2, dk=64, dv=64, C=64, dtype="f32", backward=False, seed=0),
    1: dict(name="c1_400M_bf16_fwd", B=8, T=2048, H=8, dk=128, dv=128, C=64, dtype="bf16", backward=False, seed=1),
    2: dict(name="c2_1p3B_bf16_fwd", B=4, T=4096, H=16, dk=128, dv=128, C=64, dtype="bf16", backward=False,
            seed=2, s0_std=0.02),
    3: dict(name="c3_1p3B_bf16_fwdbwd", B=4, T=4096, H=16, dk=128, dv=128, C=64, dtype="bf16", backward=True,
            seed=3, s0_std=0.02),
    4: dict(name="c4_1p3B_long_bf16_fwdbwd", B=1, T=32768, H=16, dk=128, dv=128, C=64, dtype="bf16",
            backward=True, seed=4, alpha_logit_mean=3.0, mu_logit_mean=2.0),
}


def generate(w: Workload) -> Workload:
    """Fill w.arrays with float32 numpy arrays (already bf16-representable where dtype == 'bf16').

    Draw order is fixed: q, k, v, beta logits, alpha logits, mu logits, [eta logits], S0, dO.
    """
    rng = np.random.default_rng(w.seed)
    B, T, H, dk, dv = w.B, w.T, w.H, w.dk, w.dv
    rnd = bf16_round if w.dtype == "bf16" else (lambda a: np.ascontiguousarray(a, dtype=np.float32))

    def normal(shape):
        return rng.standard_normal(shape, dtype=np.float32)

    def l2n(x):
        n = np.sqrt((x.astype(np.float64) ** 2).sum(-1, keepdims=True))
        return (x / np.maximum(n, 1e-12)).astype(np.float32)

    a = {}
    a["q"] = rnd(l2n(normal((B, T, H, dk))))
    a["k"] = rnd(l2n(normal((B, T, H, dk))))
    a["v"] = rnd(normal((B, T, H, dv)))
    a["beta"] = _sigmoid(normal((B, T, H))).astype(np.float32)
    a["alpha"] = _sigmoid(normal((B, T, H)) + np.float32(w.alpha_logit_mean)).astype(np.float32)
    mu = _sigmoid(normal((B, T, H)) + np.float32(w.mu_logit_mean))
    a["mu"] = np.maximum(mu, math.exp(w.log_mu_min)).astype(np.float32)
    if w.with_eta:
        a["eta"] = (np.tanh(normal((B, T, H)).astype(np.float64)) + 1.0).astype(np.float32)
    else:
        a["eta"] = None
    if w.s0_std > 0:
        a["S0"] = (normal((B, H, dk, dv)) * np.float32(w.s0_std)).astype(np.float32)
    else:
        a["S0"] = None
    a["M0"] = None
    if w.backward:
        a["dO"] = rnd(normal((B, T, H, dv)))
    w.arrays = a
    return w


def config(idx: int, **overrides) -> Workload:
    """Workload for measurement configuration `idx` (0..4); overrides may shrink it for tests."""
    kw = dict(CONFIGS[idx])
    kw.update(overrides)
    return generate(Workload(**kw))


def custom(**kw) -> Workload:
    """A free-form workload for tests (ragged sizes, eta, gate extremes...)."""
    kw.setdefault("name", "custom")
    kw.setdefault("C", 64)
    kw.setdefault("dtype", "f32")
    kw.setdefault("backward", False)
    kw.setdefault("seed", 0)
    return generate(Workload(**kw))


def to_device(w: Workload, device="cuda"):
    """The workload's arrays as torch tensors on `device` (q, k, v, dO in the storage dtype: the values are
    representable, so the conversion is exact; everything else fp32)."""
    import torch
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    t = {}
    for name, arr in w.arrays.items():
        if arr is None:
            t[name] = None
        elif name in ("q", "k", "v", "dO"):
            t[name] = torch.from_numpy(arr).to(device=device, dtype=dt)
        else:
            t[name] = torch.from_numpy(arr).to(device)
    return t
