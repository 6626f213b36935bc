"""SLA2 attention forward pass for MI355X (gfx950): hand-written HIP kernels
behind a C ABI (libsla2.so), with a thin ctypes binding.

`workloads` (synthetic inputs) is importable without the built library; the
binding in `api` raises at call time if the library is missing - there is no
CPU fallback.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "api"]


def __getattr__(name):
    if name == "api":
        import importlib
        return importlib.import_module(".api", __name__)
    raise AttributeError(name)
