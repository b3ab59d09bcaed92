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
    assert lib.mdn_workspace_bytes(ctypes.byref(shape(C=32)), 0, ctypes.byref(n)) == -2
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
