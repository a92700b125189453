"""MI355X-native chunk-sparse expert FFN (BlockFFN, Sec. 3.3 "Acceleration Kernels").

The package holds the HIP kernels behind a C-ABI shared library (``csrc/``), a thin
ctypes binding with the same entry-point names (``binding``), the build step
(``build``) and the seeded synthetic input generators (``workloads``).  Importing the
package loads nothing native; ``binding.lib()`` loads the shared library on first
use and raises if it has not been built.
"""

__all__ = ["binding", "build", "workloads"]
