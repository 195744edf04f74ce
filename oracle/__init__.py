"""CPU oracle for the Q-GaLore per-matrix optimizer step.

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64 restatement of
what the method computes, written from the paper.  It shares no code with the
HIP library and must never be imported by the product package; only the test
suite, the smoke check and the benchmark's CPU-baseline leg may use it.
"""
