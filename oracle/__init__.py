"""CPU oracle of the SirLLM retention step -- test infrastructure, not part of the product.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package.
"""
