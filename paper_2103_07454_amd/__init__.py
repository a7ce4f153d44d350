"""EventGraD per-iteration parameter path on MI355X (gfx950).

Sub-modules:
  inputs  -- seeded synthetic workloads (tensor shape lists, initial parameters,
             the five benchmark configurations).  Holds none of the method's
             arithmetic; it feeds both the HIP path and the test oracle.
  evg     -- thin ctypes binding over the C-ABI library ``libevg.so``
             (evg_init / evg_step / evg_stats ...).  Imported lazily so that
             ``inputs`` can be used without the HIP library being built.
"""

__all__ = ["inputs", "evg"]


def __getattr__(name):
    if name in ("inputs", "evg"):
        import importlib
        return importlib.import_module(f"{__name__}.{name}")
    raise AttributeError(name)
