"""MI355X-native BiGLA token mixer + 2D gating locality injection (ViG hot path).

`workloads` draws the seeded synthetic inputs; `binding` is the thin ctypes layer over the
C-ABI library of hand-written gfx950 kernels (built in-tree by `__graft_entry__.build()`).
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib

        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
