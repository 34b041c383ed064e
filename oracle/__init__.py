"""CPU oracle for the batched Themis evaluator -- test infrastructure only.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the product path never does.
"""
