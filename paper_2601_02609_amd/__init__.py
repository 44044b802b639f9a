"""libcce for MI355X: fused LM-head projection + token-level cross-entropy.

The package holds the HIP sources (``csrc/``), the build helper, the ctypes
binding of the C ABI declared in ``include/cce.h`` and the seeded synthetic
workload generator.  Nothing is imported eagerly: ``inputs`` is pure NumPy and
usable without a GPU, ``binding`` loads the shared library on first use and
raises if it is missing.
"""

__all__ = ["inputs", "binding", "build"]
__version__ = "0.1.0"
