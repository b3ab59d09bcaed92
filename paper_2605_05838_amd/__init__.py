"""MI355X-native Momentum DeltaNet (MDN) chunkwise forward / backward and recurrent step.

`binding` is the thin ctypes layer over the C-ABI library built from `csrc/`; `synth`
generates the seeded synthetic workloads.  Nothing here falls back to a CPU path: if the
HIP library is missing or no GPU is present the calls raise.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib

        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
