"""MI355X-native TR-Jacobi verify step (tree-verified Jacobi decoding, section
"TR-Jacobi Decoding" of the paper): thin Python binding over the C-ABI library built
from the HIP kernels in ``csrc/``.  The library is loaded on first use of the binding
(``paper_2406_17404_amd.binding``); importing the package or its input generator does
not need a GPU."""

__all__ = ["inputs", "binding"]
