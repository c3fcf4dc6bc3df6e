"""CPU oracle of the cache-enabled embedding step: test infrastructure, not product code.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this package.
"""
