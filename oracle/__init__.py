"""CPU oracle for the Hanayo per-rank hot path.  TEST INFRASTRUCTURE ONLY.

Everything under this package is a plain, slow, readable reference that the
tests, the smoke check and the benchmark's cpu_baseline leg compare the HIP
library against.  Nothing in the product package may import it, and it
imports nothing from the product package.

  schedule.py  wave placement, the per-rank F/B order, stash planning
  replay.py    brute-force replay checker for any set of per-rank lists
  block.py     transformer block / chunk forward and backward (numpy, fp64)
"""
