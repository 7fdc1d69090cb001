"""CPU oracle for the micro-rotated FP4 path.  TEST INFRASTRUCTURE ONLY.

Nothing in the product package may import this.  Tests, the smoke check and the benchmark's
CPU-baseline leg are the only callers.
"""
