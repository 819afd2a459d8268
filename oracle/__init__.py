"""CPU oracle: test infrastructure, not product code.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package.  It
shares nothing with the HIP path (no kernels, headers, helpers or constants); the only module both
sides use is the seeded input generator, which holds none of the method's arithmetic.
"""
