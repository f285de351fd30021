"""rwkvq: weight-only-quantized linear layers (scalar- or vector-quantized per
matrix) as hand-written HIP kernels for gfx950 behind a C-ABI library.

Submodules (nothing is imported eagerly, so the seeded input generators can be
used without the GPU library being present):

  synth    seeded synthetic workloads (no arithmetic of the method in it)
  binding  ctypes binding of librwkvq.so (same names as include/rwkvq.h)
  build    hipcc driver that compiles csrc/ into librwkvq.so
"""

__all__ = ["synth", "binding", "build"]
