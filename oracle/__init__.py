"""CPU oracle of the unfused, unpruned residual-network inference path.

TEST INFRASTRUCTURE ONLY.  The GPU library never imports this package; only
tests, the smoke check and the benchmark's CPU-baseline leg may.
"""
