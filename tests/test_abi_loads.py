"""CPU checks of the boundary: the library loads, exports every symbol include/mdn.h declares,
and the host-side entry points (no device access) validate their arguments."""
import ctypes
import os
import re

import pytest

from paper_2605_05838_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mdn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mdn_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree_on_the_export_list():
    assert declared_symbols() == sorted(binding.EXPORTS)


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    for name in declared_symbols():
        assert hasattr(lib, name), name
    assert lib.mdn_version() >= 100
    assert lib.mdn_strerror(0) == b"ok"
    assert b"workspace" in lib.mdn_strerror(-4)


def shape(**kw):
    base = dict(B=2, T=128, H=3, dk=128, dv=128, C=64, dtype=0, scale=0.1)
    base.update(kw)
    return binding.MdnShape(**base)


def test_workspace_query_validates_shapes():
    lib = binding.load_library()
    n = ctypes.c_size_t(0)
    assert lib.mdn_workspace_bytes(ctypes.byref(shape()), 0, ctypes.byref(n)) == 0 and n.value > 0
    fwd = n.value
    assert lib.mdn_workspace_bytes(ctypes.byref(shape()), 1, ctypes.byref(n)) == 0 and n.value > fwd
    # a partial last chunk runs on padded copies in the workspace: more workspace than the full chunks alone
    assert lib.mdn_workspace_bytes(ctypes.byref(shape(T=100)), 0, ctypes.byref(n)) == 0
    ragged = n.value
    assert lib.mdn_workspace_bytes(ctypes.byref(shape(T=64)), 0, ctypes.byref(n)) == 0 and ragged > n.value
    assert lib.mdn_workspace_bytes(ctypes.byref(shape(T=0)), 0, ctypes.byref(n)) == -2
    assert lib.mdn_saved_states_bytes(ctypes.byref(shape(T=100)), ctypes.byref(n)) == 0
    assert n.value == 2 * 3 * 2 * 2 * 128 * 128 * 2                                           # ceil(100 / 64) chunks
    assert lib.mdn_workspace_bytes(ctypes.byref(shape(dk=96, dv=96)), 0, ctypes.byref(n)) == -2
    assert lib.mdn_workspace_bytes(ctypes.byref(shape(C=48)), 0, ctypes.byref(n)) == -2
    # chunk sizes 32 and 16 (Algorithm 1): every chunk runs as a 64-token tile, so 2x / 4x the chunks' workspace plus
    # the padded copies of the tokens; the kept states follow the number of chunks
    for C in (32, 16):
        assert lib.mdn_workspace_bytes(ctypes.byref(shape(C=C)), 0, ctypes.byref(n)) == 0 and n.value > (64 // C) * fwd
        assert lib.mdn_saved_states_bytes(ctypes.byref(shape(C=C)), ctypes.byref(n)) == 0
        assert n.value == 2 * 3 * (128 // C) * 2 * 128 * 128 * 2
    assert lib.mdn_workspace_bytes_varlen(ctypes.byref(shape(B=1, C=32)), (ctypes.c_int32 * 2)(0, 128), 1, 0, ctypes.byref(n)) == -2
    assert lib.mdn_workspace_bytes(ctypes.byref(shape(dtype=7)), 0, ctypes.byref(n)) == -3
    assert lib.mdn_workspace_bytes(ctypes.byref(shape()), 0, None) == -1
    assert lib.mdn_workspace_bytes(None, 0, ctypes.byref(n)) == -1
    assert lib.mdn_saved_states_bytes(ctypes.byref(shape()), ctypes.byref(n)) == 0
    assert n.value == 2 * 3 * 2 * 2 * 128 * 128 * 2
    assert lib.mdn_saved_operands_bytes(ctypes.byref(shape()), ctypes.byref(n)) == 0 and n.value > 0
    # fp32 storage doubles every stored intermediate; the coefficient block and the two state buffers that
    # carry S, M between segments of a split call are fp32 in both modes
    fixed = 4 * 8 * 64 * 2 * 3 * 2 + 2 * (3 * 2 * 128 * 128 * 4 + 256)
    assert binding.workspace_bytes(shape(dtype=1), 0) > 1.9 * (fwd - fixed)


def test_entry_points_reject_null_and_misaligned_pointers_before_touching_a_device():
    lib = binding.load_library()
    s = shape()
    null = [None] * 17
    assert lib.mdn_chunk_fwd(ctypes.byref(s), *null[:15], None, 0, None) == -1
    assert lib.mdn_recurrent_step(ctypes.byref(s), *[None] * 10, None) == -1
    good = ctypes.c_void_p(4096)
    bad = ctypes.c_void_p(4098)
    args = [good, good, good, good, good, good, None, None, None, bad, None, None, None, None, None, good, 1 << 40,
            None]
    assert lib.mdn_chunk_fwd(ctypes.byref(s), *args) == -5
    args[9] = good
    args[16] = 16
    assert lib.mdn_chunk_fwd(ctypes.byref(s), *args) == -4


def test_cpu_tensors_are_refused():
    import torch
    x = torch.zeros(1, 64, 1, 64)
    g = torch.zeros(1, 64, 1)
    with pytest.raises(binding.MdnError):
        binding.mdn_chunk_fwd(x, x, x, g, g, g)


def test_varlen_workspace_query_validates_the_offsets():
    lib = binding.load_library()
    n = ctypes.c_size_t(0)
    cu = lambda *v: (ctypes.c_int32 * len(v))(*v)
    s1 = shape(B=1, T=300)
    assert lib.mdn_workspace_bytes_varlen(ctypes.byref(s1), cu(0, 100, 300), 2, 0, ctypes.byref(n)) == 0 and n.value > 0
    # enough for either way of running the batch: sequence by sequence (the longest one decides), or as one stream
    # of all T tokens with its own copies of alpha and mu
    whole = ctypes.c_size_t(0)
    assert lib.mdn_workspace_bytes(ctypes.byref(s1), 0, ctypes.byref(whole)) == 0
    assert n.value >= whole.value + 2 * 300 * s1.H * 4
    first = n.value
    assert lib.mdn_workspace_bytes_varlen(ctypes.byref(s1), cu(0, 150, 300), 2, 0, ctypes.byref(n)) == 0 and n.value <= first
    assert lib.mdn_workspace_bytes_varlen(ctypes.byref(s1), cu(0, 100, 299), 2, 0, ctypes.byref(n)) == -2   # does not end at T
    assert lib.mdn_workspace_bytes_varlen(ctypes.byref(s1), cu(0, 100, 100, 300), 3, 0, ctypes.byref(n)) == -2   # empty sequence
    assert lib.mdn_workspace_bytes_varlen(ctypes.byref(s1), cu(1, 100, 300), 2, 0, ctypes.byref(n)) == -2   # does not start at 0
    assert lib.mdn_workspace_bytes_varlen(ctypes.byref(shape(B=2, T=300)), cu(0, 100, 300), 2, 0, ctypes.byref(n)) == -2
    assert lib.mdn_workspace_bytes_varlen(ctypes.byref(s1), None, 2, 0, ctypes.byref(n)) == -1


def _cpu_inputs(B=1, T=64, H=2, d=64, dtype=None):
    import torch
    dtype = dtype or torch.float32
    q = torch.zeros(B, T, H, d, dtype=dtype)
    g = torch.zeros(B, T, H)
    return dict(q=q, k=q.clone(), v=q.clone(), beta=g, alpha=g.clone(), mu=g.clone())


@pytest.mark.parametrize("bad", ["k_shape", "v_dtype", "gate_shape", "gate_dtype", "S0_shape", "eta_shape", "out_o",
                                 "workspace_small", "states_small"])
def test_binding_refuses_tensors_that_do_not_fit_q_before_any_launch(bad):
    """The C ABI trusts raw pointers, so the binding checks every tensor's shape, dtype and device against what q
    implies; the checks run before a pointer is taken (they fire on CPU tensors, with no device in reach)."""
    import torch
    t = _cpu_inputs()
    kw = {}
    if bad == "k_shape":
        t["k"] = torch.zeros(1, 64, 2, 32)
    elif bad == "v_dtype":
        t["v"] = t["v"].to(torch.bfloat16)
    elif bad == "gate_shape":
        t["alpha"] = torch.zeros(1, 63, 2)
    elif bad == "gate_dtype":
        t["mu"] = t["mu"].double()
    elif bad == "S0_shape":
        kw["S0"] = torch.zeros(1, 2, 64, 32)
    elif bad == "eta_shape":
        kw["eta"] = torch.zeros(1, 64)
    elif bad == "out_o":
        kw["out"] = {"o": torch.zeros(1, 32, 2, 64)}
    elif bad == "workspace_small":
        kw["workspace"] = torch.zeros(1024, dtype=torch.uint8)
    elif bad == "states_small":
        kw.update(save_states=True, out={"states": torch.zeros(16)})
    with pytest.raises(binding.MdnError) as e:
        binding.mdn_chunk_fwd(t["q"], t["k"], t["v"], t["beta"], t["alpha"], t["mu"], **kw)
    assert "GPU" not in str(e.value), str(e.value)      # refused for what is wrong with it, not for being a CPU tensor


def test_binding_checks_the_backward_and_the_other_entry_points_too():
    import torch
    t = _cpu_inputs()
    names = ("q", "k", "v", "beta", "alpha", "mu")
    vt = torch.zeros(1, 64, 2, 64)
    with pytest.raises(binding.MdnError, match="dO"):
        binding.mdn_chunk_bwd(*(t[k] for k in names), vt, torch.zeros(1, 64, 2, 32))
    with pytest.raises(binding.MdnError, match="dS_final"):
        binding.mdn_chunk_bwd(*(t[k] for k in names), vt, vt.clone(), dS_final=torch.zeros(1, 2, 64, 64, dtype=torch.float64))
    with pytest.raises(binding.MdnError, match=r"out\['dq'\]"):
        binding.mdn_chunk_bwd(*(t[k] for k in names), vt, vt.clone(), out={"dq": torch.zeros(1, 64, 2, 32)})
    S = torch.zeros(1, 2, 64, 64)
    with pytest.raises(binding.MdnError, match="M0"):     # the states of the recurrent step go through the same check
        binding.mdn_recurrent_step(*(t[k] for k in names), S, torch.zeros(1, 2, 64, 32))
    with pytest.raises(binding.MdnError, match="cu_seqlens"):
        binding.mdn_chunk_fwd_varlen(*(t[k] for k in names), [0, 40, 63])
    with pytest.raises(binding.MdnError, match="cu_seqlens"):
        binding.mdn_chunk_fwd_varlen(*(t[k] for k in names), [0, 40, 40, 64])
    with pytest.raises(binding.MdnError, match="S0"):     # per-sequence states: [n_seq, H, dk, dv]
        binding.mdn_chunk_fwd_varlen(*(t[k] for k in names), [0, 40, 64], S0=torch.zeros(1, 2, 64, 64))
    x = torch.zeros(1, 64, 2)
    h = torch.zeros(2)
    with pytest.raises(binding.MdnError, match="b_mu"):
        binding.mdn_gates_fwd(x, x, x, x, h, h, h, torch.zeros(3), 1.0, 1.0)
    with pytest.raises(binding.MdnError, match="x_beta"):
        binding.mdn_gates_fwd(x, x, torch.zeros(1, 64, 3), x, h, h, h, h, 1.0, 1.0)
    with pytest.raises(binding.MdnError, match="x_k"):
        binding.mdn_frontend_fwd(t["q"], torch.zeros(1, 64, 2, 32), t["v"], h)
    with pytest.raises(binding.MdnError, match="w"):
        binding.mdn_epilogue_fwd(t["q"], t["q"], torch.zeros(32))


def test_backward_workspace_for_calls_with_adjoints_of_the_final_states():
    """Such a call keeps the rounding remainders of the chunk states and chunk adjoints (16-bit storage): two more
    state-sized tensors; with 32-bit storage nothing changes."""
    plain = binding.workspace_bytes(shape(), binding.MDN_WS_BWD)
    more = binding.workspace_bytes(shape(), binding.MDN_WS_BWD_STATE_ADJOINTS)
    states = 2 * 3 * 2 * 2 * 128 * 128 * 2
    assert more == plain + 2 * states
    f32 = shape(dtype=1)
    assert binding.workspace_bytes(f32, binding.MDN_WS_BWD) == binding.workspace_bytes(f32, binding.MDN_WS_BWD_STATE_ADJOINTS)
    lib = binding.load_library()
    n = ctypes.c_size_t(0)
    assert lib.mdn_workspace_bytes(ctypes.byref(shape()), 3, ctypes.byref(n)) == -2


def test_host_side_entry_points_from_several_threads():
    """mdn_set_segments is one atomic exchange for the process and the size queries touch no shared state: threads that
    call them at the same time see consistent values (every value a call returns is one that some call has set)."""
    import threading
    lib = binding.load_library()
    want = binding.workspace_bytes(shape(), binding.MDN_WS_BWD)
    old = lib.mdn_set_segments(0)
    seen, wrong = [set() for _ in range(8)], []

    def work(i):
        n = ctypes.c_size_t(0)
        for it in range(3000):
            seen[i].add(lib.mdn_set_segments(1 + (i + it) % 7))
            if lib.mdn_workspace_bytes(ctypes.byref(shape()), 1, ctypes.byref(n)) != 0 or n.value != want:
                wrong.append(n.value)
            if lib.mdn_strerror(-4 - i % 3) is None:
                wrong.append("strerror")

    threads = [threading.Thread(target=work, args=(i,)) for i in range(8)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    last = lib.mdn_set_segments(old)
    assert not wrong
    assert set().union(*seen) <= set(range(0, 8)) and 1 <= last <= 7
    assert lib.mdn_set_segments(old) == old
