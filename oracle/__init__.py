"""Test infrastructure only: the slow fp64 CPU oracle for FlashMask attention.

Nothing on the product path may import this package; it exists so that the
tests, the smoke check and the benchmark's CPU-baseline leg have a plain
definition to compare the HIP kernels against.
"""
