"""MI355X-native single-loop (incremental) cascaded reductions.

``inputs``  - seeded synthetic workloads (no method arithmetic).
``binding`` - thin ctypes binding over the C-ABI library ``librf.so``
              (argument marshalling only; every step runs in HIP kernels).
The binding is imported lazily so that ``inputs`` can be used without the
built library; calling any ``rf_*`` function without it raises.
"""

__all__ = ["inputs", "binding"]


def __getattr__(name):
    if name in ("binding", "inputs"):
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
