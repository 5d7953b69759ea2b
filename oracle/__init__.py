"""CPU oracle for zero-value compression.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the product path never does and shares no code with it.
"""
