"""CPU oracle of the SpeCache decode step: test infrastructure only.

Nothing in the product package imports this; tests, the smoke check and the
benchmark's cpu_baseline leg do.
"""
