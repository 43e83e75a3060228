"""CPU oracle for the pre-gated MoE block: test infrastructure, never part of the product.

Only tests, the smoke check and the benchmark's `cpu_baseline` leg may import this package.
"""
