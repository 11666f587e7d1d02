"""fp64 CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It shares no code with the HIP library.
"""
