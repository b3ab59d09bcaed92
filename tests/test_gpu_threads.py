"""Calls from several host threads at once, each on a stream of its own (the header of the C ABI says they are safe):
shapes with few (batch, head) pairs, which the library splits into segments on its per-device second stream, so the
threads meet at the one piece of state that calls share.  Every thread's results must be bit-identical to the same
calls made alone, and the calls made alone are checked against the oracle."""
import threading

import numpy as np
import pytest
import torch

from gpu_util import host, to_dev, worst_err
from oracle import mdn_oracle as orc
from paper_2605_05838_amd import binding, synth

pytestmark = pytest.mark.gpu
NAMES = ("q", "k", "v", "beta", "alpha", "mu")
GRADS = ("dq", "dk", "dv", "dalpha", "dbeta", "dmu", "dS0", "dM0")


def fwd_bwd(w, t):
    f = binding.mdn_chunk_fwd(*(t[k] for k in NAMES), S0=t["S0"], scale=w.scale, save_vt=True, save_states=True,
                              save_operands=True)
    g = binding.mdn_chunk_bwd(*(t[k] for k in NAMES), f["vt"], t["dO"], S0=t["S0"], states=f["states"],
                              operands=f["operands"], scale=w.scale)
    return f, g


def test_concurrent_calls_from_three_threads_match_the_calls_made_alone():
    # 2 (batch, head) pairs, 32 chunks: split into 4 segments automatically; a different length per thread
    loads = [synth.custom(B=1, T=T, H=2, dk=128, dv=128, dtype="bf16", seed=300 + i, s0_std=0.1, backward=True)
             for i, T in enumerate((2048, 2112, 2304))]
    devs = [to_dev(w) for w in loads]
    alone = []
    for w, t in zip(loads, devs):
        f, g = fwd_bwd(w, t)
        torch.cuda.synchronize()
        alone.append(({k: f[k].clone() for k in ("o", "S", "M")}, {k: g[k].clone() for k in GRADS}))
    # the calls made alone against the oracle (first workload; the others differ in length only)
    a = {k: (None if v is None else v.astype(np.float64)) for k, v in loads[0].arrays.items()}
    rf = orc.forward(a["q"], a["k"], a["v"], a["alpha"], a["beta"], a["mu"], S0=a["S0"], scale=loads[0].scale)
    assert worst_err(host(alone[0][0]["o"]), rf["o"]) <= 2e-2 and worst_err(host(alone[0][0]["S"]), rf["S"]) <= 2e-2

    rounds, errors = 6, []
    start = threading.Barrier(len(loads))

    def worker(idx):
        try:
            stream = torch.cuda.Stream()  # (default priority)
            with torch.cuda.stream(stream):
                start.wait(timeout=60)
                for _ in range(rounds):
                    f, g = fwd_bwd(loads[idx], devs[idx])
                    stream.synchronize()
                    for k, ref in alone[idx][0].items():
                        if not torch.equal(f[k], ref):
                            errors.append((idx, k))
                    for k, ref in alone[idx][1].items():
                        if not torch.equal(g[k], ref):
                            errors.append((idx, k))
        except Exception as e:  # noqa: BLE001 (reported by the main thread)
            errors.append((idx, repr(e)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(len(loads))]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=100)
    assert not any(th.is_alive() for th in threads), "a worker thread did not finish"
    assert not errors, errors
