"""CPU oracle for one rank's share of TASP (test infrastructure, not product code).

Everything in this package is a plain, slow, fp64 / integer restatement of what the
paper's method computes.  It is imported only by the tests, by the smoke check and by
the benchmark's CPU-baseline leg.  It shares no code with the HIP library and never
imports it.
"""
