"""GPU parity of mdn_chunk_bwd against the oracle's token-level fp64 adjoint (through the C ABI)."""
import numpy as np
import pytest
import torch

from gpu_util import fmt_errs, gather_pairs, host, rel_err, rms_rel_err, select_pairs, to_dev, worst_err
from oracle import mdn_oracle as orc
from paper_2605_05838_amd import binding, synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
GRADS = ("dq", "dk", "dv", "dalpha", "dbeta", "dmu", "deta", "dS0", "dM0")


def run_fwd_bwd(w, t, dS_final=None, dM_final=None, save_states=False, save_operands=False):
    f = binding.mdn_chunk_fwd(t["q"], t["k"], t["v"], t["beta"], t["alpha"], t["mu"], eta=t["eta"], S0=t["S0"],
                              M0=t["M0"], scale=w.scale, save_vt=True, save_states=save_states,
                              save_operands=save_operands)
    g = binding.mdn_chunk_bwd(t["q"], t["k"], t["v"], t["beta"], t["alpha"], t["mu"], f["vt"], t["dO"], eta=t["eta"],
                              S0=t["S0"], M0=t["M0"], states=f["states"], operands=f["operands"], dS_final=dS_final,
                              dM_final=dM_final, scale=w.scale, want_deta=True)
    torch.cuda.synchronize()
    return f, g


def check_bwd(w, pairs=None, final_adjoints=False, save_states=False, save_operands=False, adjoint_std=1.0):
    t = to_dev(w)
    dSf = dMf = None
    if final_adjoints:
        gen = torch.Generator(device="cpu").manual_seed(99)
        dSf = (torch.randn((w.B, w.H, w.dk, w.dv), generator=gen) * adjoint_std).cuda()
        dMf = (torch.randn((w.B, w.H, w.dk, w.dv), generator=gen) * adjoint_std).cuda()
    f, g = run_fwd_bwd(w, t, dSf, dMf, save_states, save_operands)
    if pairs is None:
        pairs = [(b, h) for b in range(w.B) for h in range(w.H)]
    a = select_pairs(w, pairs)
    ref = orc.backward(a["q"], a["k"], a["v"], a["alpha"], a["beta"], a["mu"], a["dO"], eta=a["eta"], S0=a["S0"],
                       M0=a["M0"], dS_T=None if dSf is None else gather_pairs(host(dSf), pairs, True),
                       dM_T=None if dMf is None else gather_pairs(host(dMf), pairs, True), scale=w.scale)
    errs = {}
    for name in GRADS:
        x = gather_pairs(host(g[name]), pairs, is_state=name in ("dS0", "dM0"))
        errs[name] = (rel_err(x, ref[name]), rms_rel_err(x, ref[name]))
    print(w.name, "max-normalised/rms-relative", fmt_errs(errs), flush=True)
    for name, e in errs.items():
        assert max(e) <= TOL[w.dtype], (w.name, name, e)
    return errs


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d", [64, 128])
def test_small_backward_all_gradients(dtype, d):
    w = synth.custom(B=2, T=256, H=2, dk=d, dv=d, dtype=dtype, seed=31, with_eta=True, s0_std=0.3, backward=True)
    rng = np.random.default_rng(6)
    w.arrays["M0"] = (rng.standard_normal((2, 2, d, d)) * 0.2).astype(np.float32)
    check_bwd(w, final_adjoints=True)


def test_single_chunk_backward_f32():
    w = synth.custom(B=1, T=64, H=1, dk=64, dv=64, dtype="f32", seed=32, backward=True)
    check_bwd(w)


def test_backward_with_states_saved_by_the_forward_equals_reconstruction():
    w = synth.custom(B=1, T=320, H=2, dk=128, dv=128, dtype="bf16", seed=33, backward=True, s0_std=0.1)
    t = to_dev(w)
    _, g1 = run_fwd_bwd(w, t, save_states=False)
    _, g2 = run_fwd_bwd(w, t, save_states=True)
    for name in GRADS:
        assert torch.equal(g1[name], g2[name]), name      # the rebuilt states are bit-identical
    check_bwd(w, save_states=True)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64), ("bf16", 64), ("f32", 128)])
def test_backward_with_operands_kept_by_the_forward_equals_recomputation(dtype, d):
    w = synth.custom(B=1, T=192, H=2, dk=d, dv=d, dtype=dtype, seed=35, backward=True, s0_std=0.1, with_eta=True)
    t = to_dev(w)
    f1, g1 = run_fwd_bwd(w, t)
    f2, g2 = run_fwd_bwd(w, t, save_states=True, save_operands=True)
    for name in ("o", "S", "M", "vt"):
        assert torch.equal(f1[name], f2[name]), name
    for name in GRADS:
        assert torch.equal(g1[name], g2[name]), name      # same operands, same arithmetic: bit-identical
    check_bwd(w, save_states=True, save_operands=True)


def test_backward_mu_zero_and_beta_zero_f32():
    w = synth.custom(B=1, T=128, H=2, dk=64, dv=64, dtype="f32", seed=34, backward=True)
    w.arrays["mu"][:, ::3] = 0.0
    w.arrays["beta"][:, 7] = 0.0
    check_bwd(w, final_adjoints=True)


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,d,T,nseg", [("bf16", 128, 1280, 4), ("f32", 64, 832, 3), ("bf16", 64, 1024, 16)])
def test_split_into_segments_on_two_streams_equals_the_unsplit_call(dtype, d, T, nseg):
    """Splitting the sequence into segments (chunk-parallel kernels beside the scans, states carried across the
    boundaries in fp32) must not change a single bit of any output, forward or backward."""
    import torch
    w = synth.custom(B=1, T=T, H=2, dk=d, dv=d, dtype=dtype, seed=36, backward=True, s0_std=0.1, with_eta=True)
    t = to_dev(w)
    dSf = torch.randn_like(t["S0"]) * 0.1
    dMf = torch.randn_like(t["S0"]) * 0.1

    def run():
        f = binding.mdn_chunk_fwd(t["q"], t["k"], t["v"], t["beta"], t["alpha"], t["mu"], eta=t["eta"], S0=t["S0"],
                                  M0=t["M0"], scale=w.scale, save_vt=True, save_states=True, save_operands=True)
        g = binding.mdn_chunk_bwd(t["q"], t["k"], t["v"], t["beta"], t["alpha"], t["mu"], f["vt"], t["dO"], eta=t["eta"],
                                  S0=t["S0"], M0=t["M0"], states=f["states"], operands=f["operands"], dS_final=dSf,
                                  dM_final=dMf, scale=w.scale, want_deta=True, want_dstates=True)
        torch.cuda.synchronize()
        return f, g

    old = binding.set_segments(1)
    try:
        f1, g1 = run()
        binding.set_segments(nseg)
        f2, g2 = run()
    finally:
        binding.set_segments(old)
    for name in ("o", "S", "M", "vt", "states"):
        assert torch.equal(f1[name], f2[name]), name
    for name in ("dq", "dk", "dv", "dalpha", "dbeta", "dmu", "deta", "dS0", "dM0"):
        assert torch.equal(g1[name], g2[name]), name


@pytest.mark.parametrize("dtype,d,T,keep_states,keep_operands",
                         [("f32", 64, 200, False, False), ("bf16", 128, 200, True, True), ("f32", 128, 40, False, False),
                          ("bf16", 64, 135, True, False), ("f32", 64, 200, False, True), ("bf16", 64, 40, True, True),
                          ("f32", 64, 1, True, False)])
def test_backward_of_a_sequence_length_that_is_not_a_multiple_of_the_chunk_size(dtype, d, T, keep_states, keep_operands):
    """All gradients of the T tokens given, with adjoints of the final states coming in, whether the forward kept
    its states / operands or the backward rebuilds them (the partial chunk goes first in the reverse pass and takes
    its start states from what the full chunks leave)."""
    w = synth.custom(B=2, T=T, H=2, dk=d, dv=d, dtype=dtype, seed=43, with_eta=True, s0_std=0.3, backward=True)
    rng = np.random.default_rng(9)
    w.arrays["M0"] = (rng.standard_normal((2, 2, d, d)) * 0.2).astype(np.float32)
    check_bwd(w, final_adjoints=True, save_states=keep_states, save_operands=keep_operands)


@pytest.mark.parametrize("T,nseg", [(2048 + 37, 4), (1024 + 63, 2)])
def test_partial_last_chunk_together_with_segments_on_two_streams(T, nseg):
    """The full chunks split into segments on two streams, the partial chunk after them (before them in the reverse
    pass): same results as the oracle, and as the unsplit call bit for bit."""
    w = synth.custom(B=1, T=T, H=2, dk=64, dv=64, dtype="bf16", seed=47, with_eta=True, s0_std=0.2, backward=True)
    t = to_dev(w)
    prev = binding.set_segments(1)
    try:
        f1, g1 = run_fwd_bwd(w, t, save_states=True, save_operands=True)
        binding.set_segments(nseg)
        f2, g2 = run_fwd_bwd(w, t, save_states=True, save_operands=True)
    finally:
        binding.set_segments(prev)
    for k in ("o", "S", "M", "vt"):
        assert torch.equal(f1[k], f2[k]), k
    for k in GRADS:
        assert torch.equal(g1[k], g2[k]), k
    a = {k: (None if v is None else v.astype(np.float64)) for k, v in w.arrays.items()}
    ref = orc.backward(a["q"], a["k"], a["v"], a["alpha"], a["beta"], a["mu"], a["dO"], eta=a["eta"], S0=a["S0"],
                       M0=a["M0"], scale=w.scale)
    for name in GRADS:
        assert worst_err(host(g2[name]), ref[name]) <= TOL["bf16"], name
