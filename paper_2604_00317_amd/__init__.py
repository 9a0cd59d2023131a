"""MI355X-native execution-time planner (capacity-normalized minimum-congestion multi-path
split, Jacobi multiplicative-weights iteration) behind a C ABI.

`workloads` builds seeded synthetic inputs; `binding` is the thin ctypes layer over
`libnimble_plan.so`.  The binding is imported lazily so that input generation works without the
compiled library.
"""

__all__ = ["workloads", "binding"]


def __getattr__(name):
    if name in ("binding", "workloads"):
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
