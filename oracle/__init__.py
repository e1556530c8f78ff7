"""CPU oracle for the GraSS / FactGraSS compression path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
directory; only the tests, the smoke check and the benchmark's CPU-baseline
leg do.  It shares no code with the HIP path.
"""
