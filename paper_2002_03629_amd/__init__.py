"""MI355X-native Jacobi / GS-Jacobi sampling for MADE-style masked networks.

The compute lives in libjacobi_made.so (HIP, gfx950; C ABI in include/jacobi_made.h).
`binding` is a thin ctypes layer with the same entry-point names; `synth` draws the seeded
synthetic inputs.  Importing the package loads nothing; the library is loaded on first use
and its absence is an error (there is no CPU fallback).
"""
__all__ = ["binding", "synth", "build"]
