"""Test oracle for the HORA rollout path: test infrastructure, not the product.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import it.
"""
