"""GPU parity of the layer's elementwise front end and back end (mdn_frontend_*, mdn_epilogue_*) against the fp64
oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import layer_ops_oracle as lo
from paper_2605_05838_amd import binding

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}     # fp32: elementwise arithmetic and 64-lane sums; bf16: rounding of inputs and outputs


def rel(x, ref):
    return float(np.abs(x.astype(np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def _t(a, dtype):
    t = torch.from_numpy(a.astype(np.float32)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def _h(t):
    return t.float().cpu().numpy()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d", [64, 128])
def test_frontend_and_epilogue_match_the_oracle(dtype, d):
    rng = np.random.default_rng(61)
    B, T, H = 2, 203, 5
    xq, xk, xv, dq, dk, dv, o, g, dy = (rng.standard_normal((B, T, H, d)) for _ in range(9))
    dh = rng.uniform(-0.5, 0.5, H).astype(np.float32)
    w = rng.uniform(0.5, 1.5, d).astype(np.float32)
    dev = [_t(a, dtype) for a in (xq, xk, xv, dq, dk, dv, o, g, dy)]
    # the oracle sees exactly the values the kernels see (after rounding to the storage type)
    xq, xk, xv, dq, dk, dv, o, g, dy = (_h(t).astype(np.float64) for t in dev)
    dht, wt = torch.from_numpy(dh).cuda(), torch.from_numpy(w).cuda()
    f = binding.mdn_frontend_fwd(dev[0], dev[1], dev[2], dht)
    b = binding.mdn_frontend_bwd(dev[0], dev[1], dev[2], dht, dev[3], dev[4], dev[5])
    y = binding.mdn_epilogue_fwd(dev[6], dev[7], wt)
    e = binding.mdn_epilogue_bwd(dev[6], dev[7], wt, dev[8])
    torch.cuda.synchronize()
    rf = lo.frontend_forward(xq, xk, xv, dh)
    rb = lo.frontend_backward(xq, xk, xv, dh, dq, dk, dv)
    tol = TOL[dtype]
    for k in ("q", "k", "v"):
        assert rel(_h(f[k]), rf[k]) <= tol, k
    for k in ("dx_q", "dx_k", "dx_v"):
        assert rel(_h(b[k]), rb[k]) <= tol, k
    assert rel(_h(b["dd"]), rb["dd"]) <= max(tol, 1e-4)
    assert rel(_h(y), lo.epilogue_forward(o, g, w)) <= tol
    re_ = lo.epilogue_backward(o, g, w, dy)
    assert rel(_h(e["do"]), re_["do"]) <= tol and rel(_h(e["dg"]), re_["dg"]) <= tol
    assert rel(_h(e["dw"]), re_["dw"]) <= max(tol, 1e-4)
