"""GPU parity over a seeded sweep of shapes and call options: odd batch and head counts (workgroup placement with
B*H not a multiple of the 8 dies), lengths around the chunk boundaries, both storage types and head sizes, with and
without kept states / operands, initial states and adjoints of the final states.  The forward outputs
(o, V~, final states) and every gradient are compared with the fp64 oracle."""
import random

import numpy as np
import pytest

from paper_2605_05838_amd import synth
from test_gpu_backward import check_bwd
from test_gpu_forward import check_fwd

pytestmark = pytest.mark.gpu


def cases(seed, n):
    rnd = random.Random(seed)
    out = []
    for case in range(n):
        B = rnd.choice([1, 2, 3]); H = rnd.choice([1, 2, 3, 5]); d = rnd.choice([64, 128])
        dtype = rnd.choice(["f32", "bf16"])
        T = rnd.choice([rnd.randint(1, 63), 64, 65, rnd.randint(66, 400), 191, 192, 193, rnd.randint(401, 900)])
        out.append((case, B, T, H, d, dtype, rnd.random() < 0.5, rnd.random() < 0.5, rnd.random() < 0.5,
                    rnd.random() < 0.5, rnd.random() < 0.6, rnd.random() < 0.5))
    return out


@pytest.mark.parametrize("case,B,T,H,d,dtype,keep_states,keep_operands,final_adjoints,with_eta,with_s0,with_m0",
                         cases(7, 14))
def test_seeded_shape_sweep(case, B, T, H, d, dtype, keep_states, keep_operands, final_adjoints, with_eta, with_s0,
                            with_m0):
    kw = dict(B=B, T=T, H=H, dk=d, dv=d, dtype=dtype, seed=2000 + case, backward=True, with_eta=with_eta)
    if with_s0:
        kw["s0_std"] = 0.2
    w = synth.custom(**kw)
    if with_m0:
        w.arrays["M0"] = (np.random.default_rng(case).standard_normal((B, H, d, d)) * 0.2).astype(np.float32)
    check_fwd(w)  # o, V~ and the final states of the inference-mode forward
    check_bwd(w, final_adjoints=final_adjoints, save_states=keep_states, save_operands=keep_operands)
