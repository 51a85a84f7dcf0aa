"""CPU oracle of the retrieval-attention path: test infrastructure only.

Nothing in the product package imports this; only tests, the smoke check and
the benchmark's cpu_baseline leg do.
"""
