"""MI355X-native matmuls of Hadamard Domain Quantized Training (HDQT).

`binding` wraps the C ABI of libhdqt.so (include/hdqt.h); `workloads` draws the
seeded synthetic inputs; `build` compiles the HIP sources for gfx950.  Importing
the package loads nothing; the library is opened on first use and its absence
is an error (no fallback).
"""
__all__ = ["binding", "workloads", "build"]
