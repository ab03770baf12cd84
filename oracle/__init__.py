"""CPU oracle for the MARS verification pass -- test infrastructure only.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the product path (the HIP library and its binding) never does.
"""
