"""CPU oracle for Invariant Point Attention -- test infrastructure only.

Nothing in the product package imports this; only tests, the smoke check and
the benchmark's CPU-baseline leg do.
"""
