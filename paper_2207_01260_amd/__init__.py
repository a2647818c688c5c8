"""MI355X-native hot path of compiler-informed channel pruning (CPrune).

The package holds the HIP kernels and C-ABI library (``csrc/``), a thin ctypes
binding with the same entry-point names (``binding``), the host-side pruning /
inference drivers built on those calls (``pipeline``) and the seeded synthetic
workload generators (``synth``).  Importing the package loads nothing native:
``binding.lib()`` loads the shared library on first use and raises if it has
not been built.
"""

__all__ = ["binding", "pipeline", "synth"]
