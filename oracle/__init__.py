"""CPU oracle for the rollout hot path -- test infrastructure only.

Nothing in the product imports this package.  Tests, the smoke check and the
CPU-baseline leg of the benchmark are its only callers.
"""
