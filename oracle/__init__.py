"""CPU oracle for spatio-temporal Monarch attention (test infrastructure only).

Nothing in the product path may import this package: it exists so that the
tests, the smoke check and the benchmark's CPU-baseline leg have an
independent statement of what the HIP kernels must compute.
"""
