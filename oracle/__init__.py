"""CPU oracle for sparse 3-D convolution (test infrastructure only).

Nothing in the product package may import this package: it exists so that the
tests, the smoke check and the benchmark's cpu_baseline leg can compare the
HIP path with an independent, slow, plainly written float64 implementation.
"""
