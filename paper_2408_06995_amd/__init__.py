"""MI355X-native quantized U-Net layers on low-bitwidth floating-point codes (arxiv 2408.06995).

`binding` holds the ctypes wrappers of the C ABI in include/fpq.h (same function names);
`synth` holds the seeded synthetic workloads.  Importing this package does not load the shared
library; the first call into `binding` does, and fails loudly if libfpq.so was not built.
"""
__all__ = ["binding", "synth"]
