"""fp64 CPU oracle of the decoder hot path -- test infrastructure only.

Nothing in the product package may import this; only tests, the smoke check and
the benchmark's CPU-baseline leg do.
"""
