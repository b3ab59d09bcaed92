"""GPU parity of the packed variable-length entry points against the oracle run sequence by sequence."""
import numpy as np
import pytest
import torch

from gpu_util import host, to_dev, worst_err
from oracle import mdn_oracle as orc
from paper_2605_05838_amd import binding, synth

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.mark.parametrize("dtype,d,lens", [("f32", 64, (70, 128, 5, 191)), ("bf16", 128, (256, 33, 200))])
def test_packed_sequences_forward_and_backward(dtype, d, lens):
    T, H = sum(lens), 3
    w = synth.custom(B=1, T=T, H=H, dk=d, dv=d, dtype=dtype, seed=71, with_eta=True, backward=True)
    t = to_dev(w)
    n = len(lens)
    cu = np.concatenate([[0], np.cumsum(lens)]).tolist()
    rng = np.random.default_rng(3)
    S0 = (rng.standard_normal((n, H, d, d)) * 0.2).astype(np.float32)
    M0 = (rng.standard_normal((n, H, d, d)) * 0.1).astype(np.float32)
    dSf = rng.standard_normal((n, H, d, d)).astype(np.float32)
    dMf = rng.standard_normal((n, H, d, d)).astype(np.float32)
    dev = lambda a: torch.from_numpy(a).cuda()
    f = binding.mdn_chunk_fwd_varlen(t["q"], t["k"], t["v"], t["beta"], t["alpha"], t["mu"], cu, eta=t["eta"], S0=dev(S0),
                                     M0=dev(M0), scale=w.scale, save_vt=True)
    g = binding.mdn_chunk_bwd_varlen(t["q"], t["k"], t["v"], t["beta"], t["alpha"], t["mu"], f["vt"], t["dO"], cu,
                                     eta=t["eta"], S0=dev(S0), M0=dev(M0), dS_final=dev(dSf), dM_final=dev(dMf),
                                     scale=w.scale, want_deta=True)
    torch.cuda.synchronize()
    a = {k: (None if v is None else v.astype(np.float64)) for k, v in w.arrays.items()}
    tol = TOL[dtype]
    for i in range(n):
        sl = slice(cu[i], cu[i + 1])
        seq = {k: a[k][:, sl] for k in ("q", "k", "v", "alpha", "beta", "mu", "eta", "dO")}
        s0, m0 = S0[i:i + 1].astype(np.float64), M0[i:i + 1].astype(np.float64)
        rf = orc.forward(seq["q"], seq["k"], seq["v"], seq["alpha"], seq["beta"], seq["mu"], eta=seq["eta"], S0=s0, M0=m0,
                         scale=w.scale)
        assert worst_err(host(f["o"])[:, sl], rf["o"]) <= tol, (i, "o")
        assert worst_err(host(f["S"])[i:i + 1], rf["S"]) <= tol and worst_err(host(f["M"])[i:i + 1], rf["M"]) <= tol, (i, "S/M")
        rb = orc.backward(seq["q"], seq["k"], seq["v"], seq["alpha"], seq["beta"], seq["mu"], seq["dO"], eta=seq["eta"],
                          S0=s0, M0=m0, dS_T=dSf[i:i + 1].astype(np.float64), dM_T=dMf[i:i + 1].astype(np.float64),
                          scale=w.scale)
        for name in ("dq", "dk", "dv", "dalpha", "dbeta", "dmu", "deta"):
            assert worst_err(host(g[name])[:, sl], rb[name]) <= tol, (i, name)
        for name in ("dS0", "dM0"):
            assert worst_err(host(g[name])[i:i + 1], rb[name]) <= tol, (i, name)


@pytest.mark.parametrize("dtype,d,lens", [("f32", 64, (70, 128, 5, 191, 1, 64)), ("bf16", 128, (256, 33, 200, 1, 63, 65)),
                                          ("bf16", 64, (40,) * 9), ("f32", 128, (300,)),
                                          ("f32", 64, (700, 333, 64, 1, 900, 250)), ("bf16", 128, (1030, 1100))])
def test_packed_sequences_as_one_stream_of_tokens(dtype, d, lens):
    """No per-sequence states in or out: the library runs the batch as one stream with alpha = mu = 0 at the sequence
    starts.  Every sequence must come out as the oracle computes it by itself from zero states (sequence starts inside
    chunks, on chunk boundaries, sequences of one token; the two longest batches are cut in two halves that run beside
    each other on two streams), and the caller's alpha, mu must be left as they were."""
    T, H = sum(lens), 3
    w = synth.custom(B=1, T=T, H=H, dk=d, dv=d, dtype=dtype, seed=72, with_eta=True, backward=True)
    t = to_dev(w)
    n = len(lens)
    cu = np.concatenate([[0], np.cumsum(lens)]).tolist()
    al0, mu0 = t["alpha"].clone(), t["mu"].clone()
    f = binding.mdn_chunk_fwd_varlen(t["q"], t["k"], t["v"], t["beta"], t["alpha"], t["mu"], cu, eta=t["eta"],
                                     scale=w.scale, save_vt=True, want_states=False)
    g = binding.mdn_chunk_bwd_varlen(t["q"], t["k"], t["v"], t["beta"], t["alpha"], t["mu"], f["vt"], t["dO"], cu,
                                     eta=t["eta"], scale=w.scale, want_deta=True, want_state_grads=False)
    torch.cuda.synchronize()
    assert f["S"] is None and g["dS0"] is None
    assert torch.equal(al0, t["alpha"]) and torch.equal(mu0, t["mu"])
    a = {k: (None if v is None else v.astype(np.float64)) for k, v in w.arrays.items()}
    tol = TOL[dtype]
    for i in range(n):
        sl = slice(cu[i], cu[i + 1])
        seq = {k: a[k][:, sl] for k in ("q", "k", "v", "alpha", "beta", "mu", "eta", "dO")}
        rf = orc.forward(seq["q"], seq["k"], seq["v"], seq["alpha"], seq["beta"], seq["mu"], eta=seq["eta"], scale=w.scale)
        assert worst_err(host(f["o"])[:, sl], rf["o"]) <= tol, (i, "o")
        assert worst_err(host(f["vt"])[:, sl], rf["vt"]) <= tol, (i, "vt")
        rb = orc.backward(seq["q"], seq["k"], seq["v"], seq["alpha"], seq["beta"], seq["mu"], seq["dO"], eta=seq["eta"],
                          scale=w.scale)
        for name in ("dq", "dk", "dv", "dalpha", "dbeta", "dmu", "deta"):
            assert worst_err(host(g[name])[:, sl], rb[name]) <= tol, (i, name)
        # the first token's alpha, mu multiply zero states: their gradients are exactly zero
        assert float(host(g["dalpha"])[:, cu[i]].max()) == 0.0 and float(host(g["dmu"])[:, cu[i]].min()) == 0.0, i


@pytest.mark.parametrize("dtype,d,lens", [("f32", 64, (70, 128, 5, 191, 1, 64, 3, 2)), ("bf16", 128, (256, 33, 200, 1, 63, 65)),
                                          ("bf16", 64, (40,) * 9), ("f32", 128, (300,)), ("f32", 64, (7, 9)),
                                          ("f32", 64, (700, 333, 64, 1, 900, 250)), ("bf16", 128, (1030, 1100))])
def test_packed_prompts_with_final_states_of_every_sequence(dtype, d, lens):
    """Zero initial states, final states wanted (prefill of a batch of prompts): the stream form, then one batch of the
    sequences' last chunks run again from their start states.  o and every sequence's S, M against the oracle
    (sequences that end inside a chunk, on a chunk boundary, several sequences inside one chunk, a total length below
    one chunk, batches long enough to be cut in two halves that run beside each other)."""
    T, H = sum(lens), 2
    w = synth.custom(B=1, T=T, H=H, dk=d, dv=d, dtype=dtype, seed=73, with_eta=True)
    t = to_dev(w)
    n = len(lens)
    cu = np.concatenate([[0], np.cumsum(lens)]).tolist()
    f = binding.mdn_chunk_fwd_varlen(t["q"], t["k"], t["v"], t["beta"], t["alpha"], t["mu"], cu, eta=t["eta"],
                                     scale=w.scale)
    torch.cuda.synchronize()
    a = {k: (None if v is None else v.astype(np.float64)) for k, v in w.arrays.items()}
    tol = TOL[dtype]
    for i in range(n):
        sl = slice(cu[i], cu[i + 1])
        seq = {k: a[k][:, sl] for k in ("q", "k", "v", "alpha", "beta", "mu", "eta")}
        rf = orc.forward(seq["q"], seq["k"], seq["v"], seq["alpha"], seq["beta"], seq["mu"], eta=seq["eta"], scale=w.scale)
        assert worst_err(host(f["o"])[:, sl], rf["o"]) <= tol, (i, "o")
        assert worst_err(host(f["S"])[i:i + 1], rf["S"]) <= tol, (i, "S")
        assert worst_err(host(f["M"])[i:i + 1], rf["M"]) <= tol, (i, "M")
