"""GPU parity of mdn_gates_fwd / mdn_gates_bwd against the fp64 oracle of the gate parameterisation (through the C ABI)."""
import numpy as np
import pytest
import torch

from oracle import gates_oracle as go
from paper_2605_05838_amd import binding

pytestmark = pytest.mark.gpu


def _case(B, T, H, seed):
    rng = np.random.default_rng(seed)
    x = [(rng.standard_normal((B, T, H)) * 2.0).astype(np.float32) for _ in range(4)]
    par = [rng.uniform(0.2, 2.0, H).astype(np.float32), rng.standard_normal(H).astype(np.float32),
           rng.uniform(0.2, 2.0, H).astype(np.float32), rng.standard_normal(H).astype(np.float32)]
    d = [rng.standard_normal((B, T, H)).astype(np.float32) for _ in range(4)]
    return x, par, d


def rel(x, ref):
    return float(np.abs(x.astype(np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


@pytest.mark.parametrize("B,T,H,s,tau", [(2, 300, 16, 0.7, 11.3), (1, 77, 3, 1.5, 1.0), (3, 4096, 16, 0.3, 8.0)])
def test_gates_forward_and_backward_match_the_oracle(B, T, H, s, tau):
    x, par, d = _case(B, T, H, 5)
    dev = lambda a: torch.from_numpy(a).cuda()
    xs, ps, ds = [dev(a) for a in x], [dev(a) for a in par], [dev(a) for a in d]
    f = binding.mdn_gates_fwd(*xs, *ps, s, tau)
    g = binding.mdn_gates_bwd(*xs, *ps, s, tau, *ds)
    torch.cuda.synchronize()
    rf = go.forward(*x, *par, s, tau)
    rb = go.backward(*x, *par, s, tau, *d)
    for k in ("alpha", "beta", "mu", "eta"):
        assert rel(f[k].cpu().numpy(), rf[k]) <= 1e-5, k          # fp32 elementwise arithmetic
    for k in ("dx_alpha", "dx_mu", "dx_beta", "dx_eta"):
        assert rel(g[k].cpu().numpy(), rb[k]) <= 1e-5, k
    dp = g["dparams"].cpu().numpy()
    for i, k in enumerate(("da_alpha", "db_alpha", "da_mu", "db_mu")):
        assert rel(dp[i], rb[k]) <= 1e-4, k                        # fp32 sums over B*T terms in atomic order


def test_gates_feed_the_chunkwise_forward():
    """The gates this front end produces are in the ranges the chunkwise path is built for: run it on them."""
    from paper_2605_05838_amd import synth
    from gpu_util import to_dev
    w = synth.custom(B=1, T=128, H=2, dk=64, dv=64, dtype="f32", seed=3)
    t = to_dev(w)
    x, par, _ = _case(1, 128, 2, 9)
    dev = lambda a: torch.from_numpy(a).cuda()
    gts = binding.mdn_gates_fwd(*[dev(a) for a in x], *[dev(a) for a in par], 0.8, 4.0)
    r = binding.mdn_chunk_fwd(t["q"], t["k"], t["v"], gts["beta"], gts["alpha"], gts["mu"], eta=gts["eta"], scale=w.scale)
    torch.cuda.synchronize()
    from oracle import mdn_oracle as orc
    a = {k: v.astype(np.float64) for k, v in w.arrays.items() if v is not None and k in ("q", "k", "v")}
    ref = orc.forward(a["q"], a["k"], a["v"], gts["alpha"].cpu().numpy().astype(np.float64),
                      gts["beta"].cpu().numpy().astype(np.float64), gts["mu"].cpu().numpy().astype(np.float64),
                      eta=gts["eta"].cpu().numpy().astype(np.float64), scale=w.scale)
    assert rel(r["o"].cpu().numpy(), ref["o"]) <= 1e-4
