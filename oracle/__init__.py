"""CPU oracle for the BlockPerm-SJLT sketch apply.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
directory; only the tests, the smoke check and the benchmark's CPU-baseline
leg use it.  It is slow on purpose: float64, explicit sparse matrix, no
blocking or fusion.  It shares no code with the HIP path.
"""
