"""Brute-force one-sided (Hestenes) Jacobi SVD, pure numpy, fp64.

Step 5 of Algorithm 1 decomposes the small matrix B with a Jacobi solver
(method section, note on step 5: plane rotations, quadratic convergence, a
handful of sweeps).  The paper gives no stopping rule or pair order, so this
oracle takes the plainest form: cyclic sweeps over every column pair (p < q),
one rotation at a time, until a whole sweep finds every pair orthogonal to
    |a_p . a_q| <= tol * ||a_p|| * ||a_q||.
Rotation by the textbook stable formula (Golub & Van Loan, one-sided Jacobi):
    zeta = (beta - alpha) / (2 gamma),  t = sign(zeta) / (|zeta| + sqrt(1 + zeta^2)),
    c = 1 / sqrt(1 + t^2),  s = c t.
It is only meant for inputs up to about 64 x 64.
"""
import numpy as np


def jacobi_svd(M, tol=None, max_sweeps=60):
    """Full SVD  M = X diag(sigma) W^T  of an r x c matrix with r >= c.

    Returns (X r x c, sigma c, W c x c, sweeps), sigma descending.  Columns of
    X that belong to a zero singular value are zero.
    """
    A = np.array(M, dtype=np.float64, copy=True)
    r, c = A.shape
    assert r >= c
    if tol is None:
        tol = np.finfo(np.float64).eps * np.sqrt(r)
    W = np.eye(c)
    sweeps = 0
    for sweeps in range(1, max_sweeps + 1):
        rotated = False
        for p in range(c - 1):
            for q in range(p + 1, c):
                alpha = A[:, p] @ A[:, p]
                beta = A[:, q] @ A[:, q]
                gamma = A[:, p] @ A[:, q]
                if abs(gamma) <= tol * np.sqrt(alpha * beta) or gamma == 0.0:
                    continue
                rotated = True
                zeta = (beta - alpha) / (2.0 * gamma)
                t = (1.0 if zeta >= 0 else -1.0) / (abs(zeta) + np.sqrt(1.0 + zeta * zeta))
                cs = 1.0 / np.sqrt(1.0 + t * t)
                sn = cs * t
                ap, aq = A[:, p].copy(), A[:, q].copy()
                A[:, p] = cs * ap - sn * aq
                A[:, q] = sn * ap + cs * aq
                wp, wq = W[:, p].copy(), W[:, q].copy()
                W[:, p] = cs * wp - sn * wq
                W[:, q] = sn * wp + cs * wq
        if not rotated:
            break
    sigma = np.sqrt(np.sum(A * A, axis=0))
    order = np.argsort(-sigma, kind="stable")
    sigma = sigma[order]
    A = A[:, order]
    W = W[:, order]
    X = np.zeros_like(A)
    nz = sigma > 0
    X[:, nz] = A[:, nz] / sigma[nz]
    return X, sigma, W, sweeps
