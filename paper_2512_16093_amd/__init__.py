"""MI355X-native forward pass of Sparse-Linear Attention with a low-bit
(INT8 QK^T, FP8 PV) sparse softmax branch: hand-written HIP kernels for gfx950
behind a C-ABI library, plus this thin ctypes binding.

Importing the package loads nothing; the shared library is opened on first use
(`paper_2512_16093_amd.binding.lib()`), and every call fails loudly if it is
missing.  `synth` (input generators) has no dependency on the library.
"""
__all__ = ["binding", "synth"]
