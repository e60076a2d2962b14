"""liblstm355: stacked (optionally bidirectional) LSTM inference forward pass with
sparsity masks, as hand-written HIP kernels for gfx950 behind a C ABI.

Sub-modules
  inputs   seeded synthetic workloads (numpy only; no LSTM arithmetic)
  binding  ctypes binding of the C ABI declared in include/lstm355.h
  build    hipcc driver that produces liblstm355.so in-tree

Nothing is imported eagerly so that `inputs` stays usable without the native library.
"""
__all__ = ["inputs", "binding", "build"]
