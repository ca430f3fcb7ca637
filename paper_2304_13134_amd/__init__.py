"""MI355X-native lattice forward/backward for globally normalised training
(the hot path of arXiv 2304.13134): a thin Python binding over the C-ABI HIP
library built from ``csrc/``.  The library is loaded on first use; there is no
CPU fallback."""
__all__ = ["workloads"]
