"""Float64 CPU oracle for alpha-entmax attention (test infrastructure only).

Nothing in the product package imports this; only tests, the smoke check and the
CPU-baseline leg of the benchmark do.
"""
