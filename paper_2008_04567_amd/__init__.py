"""MI355X-native forward 2-D convolution with a genetic autotuner (libwpk + ctypes binding).

``binding`` mirrors the C ABI declared in ``include/wpk.h``; ``workloads`` holds the seeded
synthetic layer shapes and tensors; ``build`` compiles the HIP library in-tree.  Importing the
package loads nothing; the library is opened on first use and its absence is an error.
"""
from . import binding, workloads  # noqa: F401

__all__ = ["binding", "workloads"]
