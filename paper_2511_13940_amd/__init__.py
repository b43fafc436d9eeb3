"""MI355X-native per-rank GEMM+reduce-scatter and all-gather+GEMM (gfx950 HIP kernels behind a C ABI).

`paper_2511_13940_amd.pk` is the ctypes binding of libpk.so; `workloads` holds
the seeded synthetic input generators.  Importing the package loads nothing;
the binding loads the library on first use and raises if it has not been built.
"""
__all__ = ["pk", "workloads"]
