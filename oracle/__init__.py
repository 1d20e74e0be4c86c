"""CPU oracle (fp64) for packed variable-length causal attention.

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg.  The GPU library never imports or links it.
"""
