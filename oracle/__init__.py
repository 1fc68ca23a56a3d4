"""CPU oracle: test infrastructure only.

Nothing in the product path (the HIP library or its Python binding) may import
this package; only tests, the smoke check and the benchmark's CPU-baseline leg do.
"""
