"""EchoKV decode hot path for MI355X (gfx950): HIP kernels behind a C ABI.

`synth` holds the seeded workload generators; `binding` is the ctypes layer
over libechokv.so (loaded on first use; there is no CPU fallback).
"""
__all__ = ["synth", "binding", "build"]
