"""The forward entry point that allocates nothing (mdn_chunk_fwd_noalloc: its workspace is a fixed array inside the
library's device image) against mdn_chunk_fwd, through the C ABI: same kernels on the same inputs, so every output
must agree bit for bit; two calls in a row, the second on a smaller input (the array keeps the first call's
contents); a shape beyond the array's size is refused before anything is launched."""
import pytest
import torch

from gpu_util import to_dev
from paper_2605_05838_amd import binding, synth

pytestmark = pytest.mark.gpu

NAMES = ("q", "k", "v", "beta", "alpha", "mu")


def both(w):
    t = to_dev(w)
    ref = binding.mdn_chunk_fwd(*(t[k] for k in NAMES), eta=t["eta"], S0=t["S0"], M0=t["M0"], scale=w.scale, save_vt=True)
    out = {"o": torch.full_like(ref["o"], 7.0), "S": torch.full_like(ref["S"], 7.0), "M": torch.full_like(ref["M"], 7.0),
           "vt": torch.full_like(ref["vt"], 7.0)}
    before = torch.cuda.memory_allocated()
    binding.mdn_chunk_fwd_noalloc(*(t[k] for k in NAMES), out, eta=t["eta"], S0=t["S0"], M0=t["M0"], scale=w.scale)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for name in ("o", "S", "M", "vt"):
        assert torch.equal(out[name], ref[name]), (w.name, name)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
def test_two_calls_in_a_row_the_second_smaller(dtype, d):
    both(synth.custom(name="first", B=2, T=1024 + 37, H=3, dk=d, dv=d, dtype=dtype, seed=71, with_eta=True, s0_std=0.2))
    both(synth.custom(name="second", B=1, T=200, H=2, dk=d, dv=d, dtype=dtype, seed=72, s0_std=0.1))


def test_a_shape_beyond_the_fixed_array_is_refused():
    import ctypes
    lib = binding.load_library()
    shape = binding.MdnShape(4, 4096, 16, 128, 128, 64, binding.MDN_DTYPE_BF16, 0.1)
    assert binding.workspace_bytes(shape, binding.MDN_WS_FWD) > (64 << 20)
    good = ctypes.c_void_p(4096)
    args = [good] * 6 + [None, None, None, good, None, None, None, None]
    assert lib.mdn_chunk_fwd_noalloc(ctypes.byref(shape), *args) == -4
    small = binding.MdnShape(1, 4096, 16, 128, 128, 64, binding.MDN_DTYPE_BF16, 0.1)
    assert binding.workspace_bytes(small, binding.MDN_WS_FWD) <= (64 << 20)
