"""Chunk sizes 16 and 32 (Algorithm 1 lists C in {16, 32, 64}) against the fp64 oracle, through the C ABI: the result
of the chunkwise algorithm does not depend on C, so every chunk size must match the token-by-token recurrence, forward
and backward, and the three chunk sizes must agree with each other to rounding."""
import numpy as np
import pytest
import torch

from gpu_util import host, to_dev, worst_err
from oracle import mdn_oracle as orc
from paper_2605_05838_amd import binding, synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
NAMES = ("q", "k", "v", "beta", "alpha", "mu")


def run(w, t, C, keep, dSf=None, dMf=None):
    f = binding.mdn_chunk_fwd(*(t[k] for k in NAMES), eta=t["eta"], S0=t["S0"], M0=t["M0"], scale=w.scale, save_vt=True,
                              save_states=keep, save_operands=keep, chunk_size=C)
    g = None
    if w.backward:
        g = binding.mdn_chunk_bwd(*(t[k] for k in NAMES), f["vt"], t["dO"], eta=t["eta"], S0=t["S0"], M0=t["M0"],
                                  states=f["states"], operands=f["operands"], dS_final=dSf, dM_final=dMf, scale=w.scale,
                                  want_deta=True, chunk_size=C)
    torch.cuda.synchronize()
    return f, g


@pytest.mark.parametrize("C", [16, 32])
def test_config0_at_smaller_chunk_sizes(C):
    w = synth.config(0)
    t = to_dev(w)
    f, _ = run(w, t, C, False)
    a = {k: (None if v is None else v.astype(np.float64)) for k, v in w.arrays.items()}
    ref = orc.forward(a["q"], a["k"], a["v"], a["alpha"], a["beta"], a["mu"], scale=w.scale)
    for name in ("o", "vt", "S", "M"):
        assert worst_err(host(f[name]), ref[name]) <= TOL["f32"], (C, name)


@pytest.mark.parametrize("dtype,d,T,C,keep", [("bf16", 128, 200, 32, True), ("bf16", 64, 333, 16, False),
                                              ("f32", 64, 130, 16, True), ("f32", 128, 96, 32, False),
                                              ("bf16", 128, 7, 16, False)])
def test_forward_and_backward_at_smaller_chunk_sizes(dtype, d, T, C, keep):
    w = synth.custom(B=2, T=T, H=3, dk=d, dv=d, dtype=dtype, seed=90 + C, with_eta=True, s0_std=0.2, backward=True)
    w.arrays["M0"] = (np.random.default_rng(3).standard_normal((2, 3, d, d)) * 0.2).astype(np.float32)
    t = to_dev(w)
    gen = torch.Generator(device="cpu").manual_seed(5)
    dSf = torch.randn((2, 3, d, d), generator=gen).cuda()
    dMf = torch.randn((2, 3, d, d), generator=gen).cuda()
    f, g = run(w, t, C, keep, dSf, dMf)
    a = {k: (None if v is None else v.astype(np.float64)) for k, v in w.arrays.items()}
    rf = orc.forward(a["q"], a["k"], a["v"], a["alpha"], a["beta"], a["mu"], eta=a["eta"], S0=a["S0"], M0=a["M0"],
                     scale=w.scale)
    rb = orc.backward(a["q"], a["k"], a["v"], a["alpha"], a["beta"], a["mu"], a["dO"], eta=a["eta"], S0=a["S0"],
                      M0=a["M0"], dS_T=host(dSf), dM_T=host(dMf), scale=w.scale)
    errs = {name: worst_err(host(f[name]), rf[name]) for name in ("o", "vt", "S", "M")}
    errs.update({name: worst_err(host(g[name]), rb[name])
                 for name in ("dq", "dk", "dv", "dalpha", "dbeta", "dmu", "deta", "dS0", "dM0")})
    print(dtype, d, T, C, {k: f"{v:.1e}" for k, v in errs.items()}, flush=True)
    for name, e in errs.items():
        assert e <= TOL[dtype], (name, e)
    # the other chunk sizes give the same tensors up to rounding
    f64, g64 = run(w, t, 64, keep, dSf, dMf)
    for name in ("o", "S", "M"):
        assert worst_err(host(f[name]), host(f64[name])) <= 2 * TOL[dtype], name
    for name in ("dq", "dalpha", "dS0"):
        assert worst_err(host(g[name]), host(g64[name])) <= 2 * TOL[dtype], name


def test_the_allocation_free_forward_takes_the_chunk_size_too():
    w = synth.custom(B=1, T=100, H=2, dk=64, dv=64, dtype="bf16", seed=77, s0_std=0.1)
    t = to_dev(w)
    ref = binding.mdn_chunk_fwd(*(t[k] for k in NAMES), S0=t["S0"], scale=w.scale, chunk_size=32)
    out = {"o": torch.empty_like(ref["o"]), "S": torch.empty_like(ref["S"]), "M": torch.empty_like(ref["M"])}
    binding.mdn_chunk_fwd_noalloc(*(t[k] for k in NAMES), out, S0=t["S0"], scale=w.scale, chunk_size=32)
    torch.cuda.synchronize()
    for name in ("o", "S", "M"):
        assert torch.equal(out[name], ref[name]), name
