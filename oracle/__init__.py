"""CPU oracle for the RoCo hot path.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path (the HIP library and its Python binding) imports
this package; only the tests, the smoke check and the benchmark's CPU-baseline
leg do.  It shares no code with the HIP path.
"""
