"""MI355X-native CoCoDC outer-synchronisation path: HIP kernels behind a C ABI.

`binding` (loaded lazily) exposes the entry points of include/cocodc.h under the same names;
`synth` holds the seeded synthetic workloads.  There is no CPU fallback: using `binding`
without the built HIP library raises.
"""
import importlib

__all__ = ["binding", "synth"]


def __getattr__(name):
    if name in __all__:
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
