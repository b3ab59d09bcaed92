"""Parity at the full sizes of the five measurement configurations, on ALL (batch, head) pairs (the oracle does a
whole configuration in seconds).  The training configurations (3, 4) run in both launch configurations: the one the
benchmark times (the forward keeps the chunk-start states and the reverse pass's operands; configuration 4 with the
automatic split into segments on two streams active) and the memory-lean one (the backward reconstructs and
recomputes)."""
import pytest

from paper_2605_05838_amd import binding, synth
from test_gpu_backward import check_bwd
from test_gpu_forward import check_fwd

pytestmark = pytest.mark.gpu


def test_config0_full():
    check_fwd(synth.config(0))


def test_config1_400M_forward():
    check_fwd(synth.config(1))


def test_config2_1p3B_forward_with_initial_state():
    check_fwd(synth.config(2))


@pytest.mark.parametrize("keep", [True, False], ids=["forward_keeps_states_and_operands", "backward_rebuilds"])
def test_config3_1p3B_forward_backward(keep):
    w = synth.config(3)
    check_fwd(w, save_states=keep, save_operands=keep)
    check_bwd(w, save_states=keep, save_operands=keep)


@pytest.mark.parametrize("keep", [True, False], ids=["forward_keeps_states_and_operands", "backward_rebuilds"])
def test_config4_long_context_forward_backward(keep):
    w = synth.config(4)
    assert binding.set_segments(0) == 0   # the automatic choice (4 segments for this shape) is what runs
    check_fwd(w, save_states=keep, save_operands=keep)
    check_bwd(w, save_states=keep, save_operands=keep)
