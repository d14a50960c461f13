"""MI355X-native SAGE hot path: Frequent Directions sketch + agreement scoring + top-m selection.

``binding`` is the thin ctypes layer over the C-ABI library declared in ``include/sage.h``; ``inputs`` holds
the seeded synthetic workloads. Nothing here falls back to a CPU implementation: if the HIP library is
missing, loading it raises.
"""
from . import inputs  # noqa: F401

__all__ = ["inputs", "binding", "build"]
