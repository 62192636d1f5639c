"""MI355X-native selective-recompute partial prefill (CacheTune online hot path).

The package holds the HIP sources (``csrc/``), the build helper (``build.py``), the ctypes
binding over the C-ABI library (``binding.py``) and the seeded synthetic input generators
(``workloads.py``).  Nothing is imported eagerly: ``workloads`` carries no method
arithmetic and must stay importable without the compiled library.
"""

__all__ = ["binding", "build", "workloads"]
