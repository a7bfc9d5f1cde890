"""MI355X-native GEMM / batched GEMM (gfx950 HIP kernels behind a C ABI).

`paper_1705_05249_amd.gemm` is the thin ctypes binding of the shared library;
`paper_1705_05249_amd.workloads` draws the seeded synthetic inputs.
Nothing is loaded at import time; the binding loads the library on first use and
raises if it has not been built.
"""
