"""fp64 CPU oracle of the FreqFormer attention path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library, its
Python binding, the timed legs of the benchmark) may import, call or link
anything in this package; only the tests, the smoke check and the benchmark's
CPU-baseline leg do.  The oracle shares no code with the HIP path.
"""
