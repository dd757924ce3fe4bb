"""CPU oracle (test infrastructure only): plain per-model operators in float64.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It shares no code with the HIP library and never imports it.
"""
