"""TEST INFRASTRUCTURE ONLY: the CPU oracle (plain, slow, independent of the GPU library).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package.
"""
