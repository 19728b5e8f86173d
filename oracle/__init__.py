"""fp64 CPU oracle for the scaled Muon step.  TEST INFRASTRUCTURE ONLY.

Nothing in the product package may import this; only tests/, the smoke check
and the bench's cpu_baseline leg do.
"""
