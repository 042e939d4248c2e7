"""fp64 CPU oracle of the EARN register-token attention path.

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's
cpu_baseline leg.  It never imports the product package, and the product package
never imports it.
"""
