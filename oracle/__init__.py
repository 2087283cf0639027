"""CPU oracle for the BubbleSpec speculative-verify step (fp64, NumPy).

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain definition that the
HIP library is checked against.  It shares no code with the HIP path and must
never be imported by the product package; only tests, the smoke check and the
benchmark's cpu-baseline leg may call it.

Modules
  decoder  target decoder forward over k+1 positions (black-box model of the
           paper's Sec. 3.3 "token-wise" + "request-wise" operations)
  accept   draft acceptance and residual resampling (Eq. 2, Eq. 3, Alg. 1)
  lookup   draft retrieval from a prompt's pool of pre-generated rollouts
           (Sec. 3.2; brute-force frequency walk)

Pin status: accept and lookup are pinned by closed forms, chi-square tests and
brute force (tests/test_oracle_*.py).  decoder is pinned only by invariants
(sequential == block pass, rotary shift invariance, GQA == repeated-MHA,
norm/softmax textbook cases) and by an independent torch-CPU module re-derived
from library primitives; absolute logit values of a random-init model have no
external reference, so those values are "parity unpinned" beyond the invariants.
"""
