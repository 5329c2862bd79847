"""fp64 CPU oracle for decode attention -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  The GPU library never does, and shares no code with it.
"""
