"""CPU oracle for the variance-based gradient compression hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; only the
test-suite, the smoke check and the benchmark's CPU-baseline leg do.  It shares
no code with the HIP path.
"""
