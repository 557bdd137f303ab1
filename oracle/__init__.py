"""CPU oracle for the NGDB training hot path.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this package: it exists so that the
tests, the smoke check and the benchmark's cpu_baseline leg have an
independent, plain definition of what one training step computes.
"""
