"""MI355X-native Dion optimizer step (arXiv 2504.05295, Algorithm "Unsharded Dion update rule").

The package holds the HIP kernels (``csrc/``), the build helper, the ctypes binding of the
C-ABI library declared in ``include/dion.h`` and the seeded synthetic-input generators.
Nothing here computes the step on the CPU: without the built HIP library every call raises.
"""

__all__ = ["inputs", "binding", "build"]
