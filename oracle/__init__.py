"""CPU oracle for the MG-WFBP merged-gradient path.  TEST INFRASTRUCTURE ONLY.

Nothing in the product package imports this; only tests/, the smoke check and
the benchmark's cpu_baseline leg do.
"""
