"""CPU oracle for the GGNN hot path -- test infrastructure only.

Nothing in the product path may import this package; only tests, the smoke check and
the CPU-baseline leg of the benchmark do.
"""
