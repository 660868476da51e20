"""Float64 CPU oracle of the Parallel Evoformer block (TEST INFRASTRUCTURE).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It shares no code with the HIP path.
"""
