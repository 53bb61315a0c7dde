"""CPU oracle for the structured-binary matrix product.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this package.  It
shares no code with the HIP library and never imports it.
"""
