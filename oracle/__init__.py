"""CPU oracle for the PAHQ / ACDC edge-ablation path.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64 numpy
implementation of what the HIP path computes.  It defines the expected
results; it shares no code with the HIP path and must never be imported by
the product package.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may use it.
"""
