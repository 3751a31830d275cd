"""MI355X-native sparse-decode hot path (score -> top-k -> resolve -> attend).

The compute lives in ``libspin.so`` (hand-written HIP for gfx950, C ABI in
``include/spin.h``); :mod:`paper_2604_26837_amd.binding` marshals torch tensors
into it.  There is no CPU fallback: using the binding without the built
library raises.
"""
from . import synth, tables  # noqa: F401  (pure numpy, no native code)

__all__ = ["synth", "tables", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
