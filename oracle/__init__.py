"""CPU oracle: plain, slow, fp64 definitions of what the MoE-layer share and the
host planners compute.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; only the
tests, the smoke check and the benchmark's CPU-baseline leg do.  It shares no code
with the HIP path.
"""
