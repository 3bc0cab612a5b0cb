"""CPU oracle for the block-diagonal Shampoo hot path (float64, numpy only).

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the tests, the smoke check and the
benchmark's `cpu_baseline` leg may import this package.  It shares no code with the
HIP library: it is a plain, slow, by-eye-checkable statement of what the path
computes, written from the paper:

  evd.py        principal inverse p-th root through the symmetric eigendecomposition
                (Section 3.1) -- the definition every other method approximates
  shampoo.py    factor accumulation, preconditioned update, one optimizer step
                (Algorithm 1), block-wise Adam grafting (Section 2.3)
  newton_db.py  Newton-Denman-Beavers coupled iteration (Section 3.3, Eqs. for
                Y_0/Z_0, E_{k-1}, Y_k/Z_k), its first-iteration shortcut, p=4 chaining,
                Frobenius / trace scaling (Section 3.4)
  chebyshev.py  coefficient fit, scalar Clenshaw, matrix Clenshaw in the plain and the
                reduced-matmul form (Appendix A)
  lowprec.py    bf16-operand emulation of the Newton-DB iteration (parity unpinned)

Pins (tests/test_oracle_*.py) tie every function to something other than itself:
closed forms, spectra chosen by construction, brute force on 2x2 / 4x4, library
routines (scipy fractional_matrix_power, numpy chebinterpolate / chebval) and the
matmul counts the paper states.
"""
