"""Float64 CPU oracle for the Tempo layers.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this package:
only the tests, the smoke check and the benchmark's CPU-baseline leg use it.
It shares no code with the HIP library and never imports it.
"""
