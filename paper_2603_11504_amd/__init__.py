"""LongFlow fused decode step for MI355X (gfx950): HIP kernels behind a C-ABI.

`workloads` holds the seeded synthetic inputs; `longflow` is the thin ctypes
binding over `liblongflow.so` (argument marshalling only).
"""
