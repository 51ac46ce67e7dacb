"""CPU oracle for the AGZO per-layer step.

TEST INFRASTRUCTURE ONLY.  Everything in this package is a plain, slow,
fp64 numpy statement of what the method computes, written from the paper
(Sec. 4.1, Alg. 1, Alg. 2, Eq. 7-10).  It shares no code with the HIP
library and must never be imported by the product path: only the test
suite, the smoke entry and the benchmark's cpu_baseline leg may use it.
"""
