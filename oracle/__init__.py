"""CPU oracle (test infrastructure, not product code).

Plain, slow, fp64 / exact-integer implementations of what the engine step computes,
written from the paper's definitions.  Only tests, the smoke check and the bench's
``cpu_baseline`` leg may import this package; the HIP path never does, and nothing here
imports the HIP path.
"""
