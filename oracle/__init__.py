"""CPU oracle for the low-bit KV-cache hot path (test infrastructure only).

Nothing in the product path may import this package: only tests, the smoke
check and the benchmark's cpu_baseline leg use it.
"""
