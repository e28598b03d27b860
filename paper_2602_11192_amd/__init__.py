"""MI355X-native MoE decode step with an offloaded-expert cache (C ABI + HIP kernels).

`binding` (the ctypes layer over libmoe_cache.so) is imported on first use so
that `build` can be imported before the library exists.
"""
from importlib import import_module

__all__ = ["binding", "build", "pool"]


def __getattr__(name):
    if name in __all__:
        return import_module("." + name, __name__)
    raise AttributeError(name)
