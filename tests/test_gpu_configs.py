"""Parity at the full sizes of the five measurement configurations, in the launch configuration the
benchmark times.  The oracle checks complete (batch, head) pairs (they are independent), sampled
across the batch and the heads; config 0 is checked in full."""
import pytest

from paper_2605_05838_amd import synth
from test_gpu_backward import check_bwd
from test_gpu_forward import check_fwd

pytestmark = pytest.mark.gpu


def test_config0_full():
    check_fwd(synth.config(0))


def test_config1_400M_forward():
    check_fwd(synth.config(1), pairs=[(0, 0), (3, 5), (7, 7), (5, 2)])


def test_config2_1p3B_forward_with_initial_state():
    check_fwd(synth.config(2), pairs=[(0, 0), (1, 9), (3, 15), (2, 4)])


def test_config3_1p3B_forward_backward():
    w = synth.config(3)
    pairs = [(0, 0), (1, 7), (3, 15), (2, 10)]
    check_fwd(w, pairs=pairs)
    check_bwd(w, pairs=pairs)


def test_config4_long_context_forward_backward():
    w = synth.config(4)
    pairs = [(0, 0), (0, 11)]
    check_fwd(w, pairs=pairs)
    check_bwd(w, pairs=pairs)
