"""instattn: decode-phase attention over a long fp16 KV cache for MI355X (gfx950).

The compute lives in a C-ABI shared library built from `csrc/` (hand-written HIP
kernels); `binding` marshals torch tensors to it and `workloads` draws the seeded
synthetic inputs.  The library is loaded on first use and a missing build is an
error: there is no CPU or PyTorch fallback.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
