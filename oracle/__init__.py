"""CPU oracle for the randomized SVD pipeline (Algorithm 1 of the paper).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this
directory; only the tests, the smoke check and the cpu_baseline leg of the
benchmark do.  Everything here is plain numpy in fp64, written out step by
step in the paper's order so it can be checked against the paper by eye.
It shares no code with the HIP path.

Pins (all in tests marked "not gpu"):
  philox.philox4x32_10      known-answer vectors of the Philox publication
  philox.philox_normal      closed form z0^2+z1^2 = -2 ln u0, moments, KS
  jacobi.jacobi_svd         closed forms (diagonal, rank one, orthogonal, 2x2)
  rsvd.small_svd (LAPACK)   brute-force Jacobi on inputs up to 64x64
  rsvd.orthonormalize       invariants ||Q^T Q - I||, ||Y - Q Q^T Y||
  rsvd.rsvd                 exact recovery of planted spectra, reduction to a
                            full SVD when l = min(m, n), Eckart-Young lower
                            bound, expectation bound of the range finder,
                            Ritz values below true ones, invariance under the
                            orthonormalisation schedule
"""
