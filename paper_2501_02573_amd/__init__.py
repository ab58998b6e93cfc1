"""MI355X-native decayed causal linear attention (chunked prefill + decode step).

The compute lives in hand-written gfx950 HIP kernels behind a C ABI
(``include/leet_attn.h``); :mod:`paper_2501_02573_amd.binding` marshals torch
tensors into that ABI.  The native library is loaded on first use of a binding
function and a missing library is an error, never a fallback.
"""
from . import workloads  # noqa: F401  (input generators; no native code needed)

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib

        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
