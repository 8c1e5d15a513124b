"""Test infrastructure only: the float64 CPU oracle of the TPLA decode path.

Nothing in the product package imports this; only tests, the smoke check and
the benchmark's CPU-baseline leg may call it.
"""
