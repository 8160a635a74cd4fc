"""MI355X-native schedule-parameterised operator kernels (arXiv 2205.13603).

`paper_2205_13603_amd.binding` is the ctypes front of the C-ABI library
declared in include/ms.h; `paper_2205_13603_amd.inputs` holds the seeded
synthetic input generators (no operator arithmetic).  Nothing is loaded at
package import time.
"""
__all__ = ["binding", "inputs", "build_lib"]
