"""CPU oracle for the blockwise-transform codec and its compressed-space operations.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; only the
tests, the smoke check and the benchmark's CPU-baseline leg do.  It shares no code
with the HIP path.
"""
