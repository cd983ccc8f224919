"""CPU oracle of the Crystal-KV decode hot path: test infrastructure only.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; it shares nothing with the HIP library.
"""
