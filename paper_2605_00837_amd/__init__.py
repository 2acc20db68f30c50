"""MI355X-native log-domain Sinkhorn (entropic optimal transport) hot path.

``workloads`` holds the seeded input generators; ``binding`` is the thin ctypes
layer over the C-ABI HIP library (imported lazily so that the generators can be
used on machines where the library is not built)."""

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name in ("binding", "workloads"):
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
