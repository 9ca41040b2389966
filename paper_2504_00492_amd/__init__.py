"""MI355X-native chunked forward of the low-rank (rank-r) delta rule of ParallelFlow
(arXiv 2504.00492, Section 3.1): hand-written HIP kernels for gfx950 behind a C ABI
(include/pf.h), plus a thin ctypes binding.  PyTorch only supplies device memory and streams.
"""
from . import synth  # noqa: F401  (pure numpy; importable without the HIP library)

__all__ = ["synth", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
