"""GPU parity of mdn_chunk_fwd / mdn_recurrent_step against the fp64 oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

from gpu_util import fmt_errs, gather_pairs, host, rel_err, rms_rel_err, select_pairs, to_dev, worst_err
from oracle import mdn_oracle as orc
from paper_2605_05838_amd import binding, synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}   # per tensor, on max |x - ref| / max |ref| and on rms(x - ref) / rms(ref)


def run_fwd(w, **kw):
    t = to_dev(w)
    r = binding.mdn_chunk_fwd(t["q"], t["k"], t["v"], t["beta"], t["alpha"], t["mu"], eta=t["eta"], S0=t["S0"],
                              M0=t["M0"], scale=w.scale, save_vt=True, **kw)
    torch.cuda.synchronize()
    return t, r


def oracle_fwd(a, scale):
    return orc.forward(a["q"], a["k"], a["v"], a["alpha"], a["beta"], a["mu"], eta=a["eta"], S0=a["S0"], M0=a["M0"],
                       scale=scale)


def check_fwd(w, pairs=None, **kw):
    """Outputs, V~ and final states against the oracle, on all (batch, head) pairs unless `pairs` names some; kw goes
    to the forward call (what it keeps for a backward)."""
    t, r = run_fwd(w, **kw)
    if pairs is None:
        pairs = [(b, h) for b in range(w.B) for h in range(w.H)]
    ref = oracle_fwd(select_pairs(w, pairs), w.scale)
    errs = {}
    for name in ("o", "vt", "S", "M"):
        x = gather_pairs(host(r[name]), pairs, name in ("S", "M"))
        errs[name] = (rel_err(x, ref[name]), rms_rel_err(x, ref[name]))
    print(w.name, "max-normalised/rms-relative", fmt_errs(errs), flush=True)
    for name, e in errs.items():
        assert max(e) <= TOL[w.dtype], (w.name, name, e)
    return errs


def test_config0_tiny_f32_forward():
    check_fwd(synth.config(0))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d", [64, 128])
def test_small_forward_with_eta_and_initial_states(dtype, d):
    w = synth.custom(B=2, T=320, H=3, dk=d, dv=d, dtype=dtype, seed=21, with_eta=True, s0_std=0.3)
    rng = np.random.default_rng(5)
    w.arrays["M0"] = (rng.standard_normal((2, 3, d, d)) * 0.2).astype(np.float32)
    check_fwd(w)


def test_single_chunk_and_mu_zero():
    w = synth.custom(B=1, T=64, H=1, dk=64, dv=64, dtype="f32", seed=22)
    w.arrays["mu"][:, ::2] = 0.0
    w.arrays["beta"][:, 5] = 0.0
    check_fwd(w)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_recurrent_step_matches_oracle_and_chunk_forward(dtype):
    w = synth.custom(B=2, T=70, H=2, dk=128, dv=128, dtype=dtype, seed=23, with_eta=True, s0_std=0.1)
    t = to_dev(w)
    S = t["S0"].clone()
    M = torch.zeros_like(S)
    # first 64 tokens in one call, the remaining 6 one token at a time (decoding)
    outs = [binding.mdn_recurrent_step(t["q"][:, :64].contiguous(), t["k"][:, :64].contiguous(),
                                       t["v"][:, :64].contiguous(), t["beta"][:, :64].contiguous(),
                                       t["alpha"][:, :64].contiguous(), t["mu"][:, :64].contiguous(), S, M,
                                       eta=t["eta"][:, :64].contiguous(), scale=w.scale)]
    for i in range(64, 70):
        sl = slice(i, i + 1)
        outs.append(binding.mdn_recurrent_step(t["q"][:, sl].contiguous(), t["k"][:, sl].contiguous(),
                                               t["v"][:, sl].contiguous(), t["beta"][:, sl].contiguous(),
                                               t["alpha"][:, sl].contiguous(), t["mu"][:, sl].contiguous(), S, M,
                                               eta=t["eta"][:, sl].contiguous(), scale=w.scale))
    torch.cuda.synchronize()
    o = torch.cat(outs, 1)
    a = {k: (None if v is None else v.astype(np.float64)) for k, v in w.arrays.items()}
    ref = oracle_fwd(a, w.scale)
    tol = 1e-5 if dtype == "f32" else 2e-2      # fp32 FMA recurrence; bf16 only rounds o
    assert worst_err(host(o), ref["o"]) <= tol
    assert worst_err(host(S), ref["S"]) <= 1e-5 and worst_err(host(M), ref["M"]) <= 1e-5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_prefill_states_hand_off_to_the_recurrent_step(dtype):
    """Prefill with the chunkwise forward, decode from the states it leaves (a block of 8 tokens in one call,
    then a single token): outputs and states equal the oracle's over the whole sequence (Fig. 1: both forms
    compute the same recurrence, so a sequence may switch from one to the other at a chunk boundary)."""
    Tp, Td = 192, 9
    w = synth.custom(B=2, T=Tp + Td, H=3, dk=128, dv=128, dtype=dtype, seed=31, with_eta=True, s0_std=0.1)
    t = to_dev(w)
    names = ("q", "k", "v", "beta", "alpha", "mu")
    cut = lambda a, b: {k: t[k][:, a:b].contiguous() for k in names + ("eta",)}
    p = cut(0, Tp)
    f = binding.mdn_chunk_fwd(*(p[k] for k in names), eta=p["eta"], S0=t["S0"], scale=w.scale)
    S, M = f["S"], f["M"]
    outs = [f["o"]]
    for a, b in ((Tp, Tp + 8), (Tp + 8, Tp + Td)):
        c = cut(a, b)
        outs.append(binding.mdn_recurrent_step(*(c[k] for k in names), S, M, eta=c["eta"], scale=w.scale))
    torch.cuda.synchronize()
    o = torch.cat(outs, 1)
    arrays = {k: (None if v is None else v.astype(np.float64)) for k, v in w.arrays.items()}
    ref = oracle_fwd(arrays, w.scale)
    tol = 1e-4 if dtype == "f32" else 2e-2
    assert worst_err(host(o)[:, Tp:], ref["o"][:, Tp:]) <= tol
    assert worst_err(host(o), ref["o"]) <= tol
    assert worst_err(host(S), ref["S"]) <= tol and worst_err(host(M), ref["M"]) <= tol


@pytest.mark.parametrize("dtype,d,T", [("f32", 64, 200), ("bf16", 128, 200), ("f32", 128, 40), ("bf16", 64, 70),
                                       ("f32", 64, 1)])
def test_sequence_length_that_is_not_a_multiple_of_the_chunk_size(dtype, d, T):
    """A partial last chunk (and a sequence shorter than one chunk) gives the outputs and final states of
    exactly the T tokens given: the padding the library adds consists of identity steps of the recurrence."""
    w = synth.custom(B=2, T=T, H=3, dk=d, dv=d, dtype=dtype, seed=41, with_eta=True, s0_std=0.3)
    rng = np.random.default_rng(8)
    w.arrays["M0"] = (rng.standard_normal((2, 3, d, d)) * 0.2).astype(np.float32)
    check_fwd(w)


@pytest.mark.parametrize("T", [63, 65, 127, 129])
def test_lengths_around_the_chunk_boundaries(T):
    w = synth.custom(B=1, T=T, H=2, dk=64, dv=64, dtype="f32", seed=53, with_eta=True, s0_std=0.3)
    check_fwd(w)


def test_sampled_kernel_timing_counts_every_launch_and_brackets_every_third():
    """mdn_profile_begin_sampled(3): an event pair around every third launch of the library; the launch counts cover
    all of them."""
    w = synth.custom(B=1, T=256, H=2, dk=64, dv=64, dtype="bf16", seed=24)
    t = to_dev(w)
    binding.profile_begin(3)
    for _ in range(6):
        binding.mdn_chunk_fwd(t["q"], t["k"], t["v"], t["beta"], t["alpha"], t["mu"], scale=w.scale)
    torch.cuda.synchronize()
    k = binding.profile_end(with_launch_counts=True)
    assert k["intra_fwd"][2] == 6 and k["scan_fwd"][2] == 6              # all launches
    assert k["intra_fwd"][1] + k["scan_fwd"][1] == 4                      # launches 0, 3, 6, 9 of 12
    assert k["intra_fwd"][1] == 2 and k["scan_fwd"][1] == 2               # (period 3 walks through the two kernels)
    assert all(k[n][0] > 0 for n in ("intra_fwd", "scan_fwd"))
    binding.profile_begin()
    binding.mdn_chunk_fwd(t["q"], t["k"], t["v"], t["beta"], t["alpha"], t["mu"], scale=w.scale)
    k = binding.profile_end()
    assert k["intra_fwd"][1] == 1 and k["scan_fwd"][1] == 1
