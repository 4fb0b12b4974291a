"""MI355X-native structured spinner (H D3 H D2 H D1 x) hot path.

``workloads`` holds seeded input recipes only.  ``binding`` is the thin ctypes
face of the C-ABI library built from ``csrc/`` (it is imported lazily so that
the input recipes stay importable on machines without the built library).
"""

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name in ("binding", "workloads"):
        import importlib

        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
