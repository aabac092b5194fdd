"""CPU fp64 oracle of the fused projection + cross-entropy path.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path imports this package;
it is used by tests/, by the smoke check and by the benchmark's cpu_baseline
leg.  It shares no code with the HIP kernels and never calls them.
"""
