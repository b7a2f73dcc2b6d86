"""MI355X-native synthesis hot path of TACOS (arXiv 2304.05301).

`binding` is the ctypes layer over the C ABI of include/tacos.h (HIP kernels for
gfx950); `topologies` generates the seeded synthetic inputs.  Nothing here falls back
to a CPU implementation.
"""
from . import topologies  # noqa: F401

__all__ = ["topologies", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
