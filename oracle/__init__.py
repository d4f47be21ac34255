"""TEST INFRASTRUCTURE: CPU oracle of the non-ideal crossbar training operations.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package; the
product path (the HIP library and its binding) never does.
"""
