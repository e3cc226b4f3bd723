"""DSSP parameter-server hot path on one MI355X: K virtual workers on K HIP
streams, hand-written gfx950 kernels behind a C ABI (include/dssp.h).

  binding   ctypes wrapper with the same names as the C entry points
  driver    runs a seeded virtual-time schedule through the library
  inputs    seeded synthetic inputs (no arithmetic of the method in there)
  buildlib  compiles csrc/*.hip into libdssp.so with hipcc for gfx950

Nothing is imported eagerly: `inputs` is usable without the built library.
"""
__all__ = ["binding", "driver", "inputs", "buildlib"]
