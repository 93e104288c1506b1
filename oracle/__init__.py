"""CPU oracle for the Trajectory Normalized Gradients hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in here is part of the product: it is a plain, slow,
single-threaded numpy / pure-Python statement of what the method computes, written from
the paper (arXiv 1901.08227), used to check the HIP library and timed as a CPU baseline.
Only the tests, the smoke check and the benchmark's CPU-baseline leg import it; it imports
nothing from the HIP package and shares no code, tables or constants with it.
"""
