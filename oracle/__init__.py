"""Test infrastructure: fp64 CPU oracle (plain C, loaded through ctypes).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this.
"""
