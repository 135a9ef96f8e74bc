"""CPU fp64 oracle for the TIDE draft-training step.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library, its
Python binding, the timed legs of the benchmark) may import this package; only
the tests, the smoke check and the benchmark's cpu_baseline leg do.
"""
