"""CPU float64 oracle of the SpecKV hot path.  TEST INFRASTRUCTURE ONLY.

Nothing on the product path may import this package; it exists so that the
tests, the smoke check and the benchmark's CPU baseline have an independent
definition of the result to compare the HIP library against.
"""
