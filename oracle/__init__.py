"""CPU checker (test infrastructure): plain fp64 loops for the fused block and its backward.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this package.
"""
