"""fp64 CPU oracle for the SK-Net / U-Net hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the GPU package imports this directory; only the
tests, the smoke check and the benchmark's cpu_baseline leg do.  It shares no code with
the HIP path.
"""
