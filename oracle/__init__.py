"""CPU fp64 oracle of the compressed linear layer.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path (the HIP library and its Python binding) may import
this package; only tests, the smoke check and the benchmark's cpu_baseline leg do.
"""
