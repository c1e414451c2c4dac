"""MI355X (gfx950) implementation of the {-1,+1} multi-branch binary matrix product.

``paper_2106_09886_amd.binding`` is the thin ctypes layer over the C-ABI library
(``include/qnn.h``); ``paper_2106_09886_amd.inputs`` draws the seeded synthetic
workloads.  Importing the package loads neither: the binding loads the HIP
library on first use and raises if it has not been built.
"""
__all__ = ["binding", "inputs", "build"]
