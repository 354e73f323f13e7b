"""CPU oracle for the error-corrected SGEMM.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the bench's `cpu_baseline` leg may import this
package.  It shares no code with the HIP path and never imports it.

  gemm      FP64 reference product and naive FP32 product (plain C, see gemm_oracle.c),
            the relative-residual metric of Eq. eval-matmul, max deviation
  split     element splits of the paper in numpy: halfhalf (Eqs. corr-elm-1 and
            corr-elm-2-1024), Markidis' unscaled halfhalf (Eq. corr-elm-2), the
            three-term BF16 split used for the full-exponent-range mode
  model     the method written out step by step with exact (FP64) accumulation
            (Eq. corr-5-1024-reduce and its BF16 analogue)

Parity status: every function here is pinned by tests/test_oracle_pins.py against
printed values, closed forms, exact integer products or brute force, except where a
docstring says "parity unpinned".
"""
