"""CPU oracle for one GPU's share of a pre-LN transformer block (test infrastructure only).

Nothing in the product path may import this package: it exists so that tests, the smoke check and
the benchmark's CPU-baseline leg have a slow, plain, independent definition to compare against.
"""
