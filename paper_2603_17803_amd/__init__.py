"""MI355X-native hot path of co-activation-aware KV-cache offloading:
score -> top-k select -> activation trace -> co-activation counts -> per-SSD request queues.

`workloads` draws seeded synthetic inputs and has no dependencies beyond numpy.
`binding` is the thin ctypes layer over the HIP library; it is imported lazily so that
input generation works on machines without the built library, while any attempt to run
the path without it raises.
"""

__all__ = ["workloads", "binding", "build"]


def __getattr__(name):
    if name in __all__:
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
