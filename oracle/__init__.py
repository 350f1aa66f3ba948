"""CPU oracle for the fused attention forward + JVP (test infrastructure only).

Nothing in the product path (the HIP library and its Python binding) may import
this package; only tests, the smoke check and the CPU-baseline leg of the bench do.
"""
