"""CPU oracle for the attention forward pass (test infrastructure only).

Nothing in the product package may import this package; only the tests, the smoke check and
the benchmark's cpu_baseline leg do.
"""
