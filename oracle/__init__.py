"""CPU oracle for the token-routed sparse FFN layer (TEST INFRASTRUCTURE ONLY).

Nothing in the product package imports this. Only tests, the smoke check and
the benchmark's cpu_baseline leg may call it.
"""
