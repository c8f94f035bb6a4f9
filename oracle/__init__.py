"""CPU oracle of the decoder hot path.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the product path (the HIP library and its binding) never does.
"""
