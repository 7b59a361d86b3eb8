"""MI355X-native exact causal multi-head attention, forward and backward.

The hot path lives in hand-written HIP kernels behind a C-ABI shared library
(``csrc/``); ``binding`` marshals arguments to it.  Nothing in this package falls
back to a CPU implementation: without the built library every call raises.
"""
from . import inputs  # noqa: F401

__all__ = ["inputs", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib

        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
