"""CPU oracle for the RNS-CKKS hot path.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the GPU library never does, and it shares no code with it.
"""
