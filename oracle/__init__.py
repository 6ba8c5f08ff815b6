"""CPU oracle for the rotated low-bit linear (test infrastructure only).

Nothing in the product imports this package; only tests, the smoke check and
the benchmark's cpu_baseline leg do.
"""
