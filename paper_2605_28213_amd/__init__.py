"""GEMM kernel lineage for MI355X (gfx950): C-ABI HIP library + thin binding.

``gemm``   -- ctypes binding of include/gemm_lineage.h (loads libgemm_lineage.so on first use)
``inputs`` -- seeded synthetic workloads (no GEMM arithmetic)
``gate``   -- the compile / correctness / profile gate and its per-variant ledger
``build``  -- hipcc build of the shared library
"""
