"""MI355X-native hot path of SpecVLM (arXiv 2508.16201): score, select,
gather_kv, decode_attn, accept -- hand-written HIP kernels for gfx950 behind a
C ABI (``include/specvlm.h``), bound with ctypes in ``binding``.

Importing the package loads nothing; the HIP library is opened on first use
and there is no fallback if it is missing.
"""
from . import synth  # noqa: F401  (seeded inputs; NumPy only)

__all__ = ["binding", "build", "synth"]


def __getattr__(name):
    if name in ("binding", "build"):
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
