"""MI355X-native Top-k + error-feedback gradient compression (the GraVAC hot path).

``binding`` wraps the C ABI of ``include/gravac.h`` (``libgravac.so``, hand-written
HIP for gfx950); ``workloads`` holds the seeded synthetic gradients.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name == "binding":
        import importlib
        return importlib.import_module(".binding", __name__)
    raise AttributeError(name)
