"""CPU oracle for choreographed attention: test infrastructure only.

Nothing in the product package imports from here; tests, the smoke check and
the benchmark's CPU-baseline leg do.
"""
