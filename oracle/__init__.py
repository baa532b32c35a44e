"""CPU oracle for the structured-decoding hot path.  TEST INFRASTRUCTURE ONLY.

Nothing in the product package imports this; the tests, the smoke check and the
benchmark's CPU-baseline leg do.
"""
