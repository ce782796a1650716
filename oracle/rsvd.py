"""Randomized k-SVD, Algorithm 1 of the paper, written out step by step (fp64).

Notation follows the paper: A is m x n, k the target rank, p the
oversampling, q the exponent of the power scheme, s = k + p (called l here
and in the rest of this repository), S the sketching matrix (Omega here).

Readings where the paper leaves a choice:
  * A^* is the transpose (real input).
  * Algorithm 1 step 2 prints Y = (A A^*)^q A S with no intermediate
    factorisation, while the notes on steps 2-3 describe QR and GEMM
    interleaved.  The oracle re-orthonormalises after every product with A or
    A^T; in exact arithmetic every such schedule spans the same range, which
    the schedule-invariance test checks.
  * Step 3 is a Householder QR (LAPACK through numpy) with explicit Q.
  * Step 5 is the SVD of the s x n matrix B (LAPACK through numpy, itself
    pinned against the brute-force Jacobi in jacobi.py); the k largest
    triplets are kept (the paper's Sigma is k x k).
"""
from types import SimpleNamespace

import numpy as np

from . import philox


def sketch(seed, n, l, dtype):
    """Step 1: Omega (n x l) ~ iid N(0,1), values representable in `dtype`, returned as fp64."""
    return philox.philox_normal(seed, n, l, dtype).astype(np.float64)


def range_product(A, X):
    """Steps 2 and 6: the plain product A X."""
    return A @ X


def adjoint_product(A, X):
    """Power scheme and step 4 (as B^T = A^T Q): the plain product A^T X."""
    return A.T @ X


def orthonormalize(Y):
    """Step 3: Q with orthonormal columns spanning range(Y), Householder QR."""
    Q, _ = np.linalg.qr(Y, mode="reduced")
    return Q


def qr_positive(Y):
    """The unique reduced QR with a non-negative diagonal of R (full column rank Y)."""
    Q, R = np.linalg.qr(Y, mode="reduced")
    sgn = np.where(np.diag(R) < 0, -1.0, 1.0)
    return Q * sgn, R * sgn[:, None]


def _cholqr2(Y):
    """CholeskyQR applied twice; only used by the schedule-invariance pin."""
    Q = Y
    for _ in range(2):
        R = np.linalg.cholesky(Q.T @ Q).T
        Q = np.linalg.solve(R.T, Q.T).T
    return Q


def small_svd(B):
    """Step 5: compact SVD of B (s x n), singular values descending."""
    return np.linalg.svd(B, full_matrices=False)


def rsvd(A, k, p, q, seed, dtype, orth="householder"):
    """Algorithm 1.  `dtype` is the precision the caller's A and Omega live in
    (fp32 inputs are up-cast exactly); all arithmetic here is fp64.

    orth: "householder" (the oracle), "cholqr2" or "none" (no intermediate
    re-orthonormalisation; final QR still done) - the last two exist for the
    schedule-invariance pin only.
    """
    A = np.asarray(A, dtype=np.float64)
    m, n = A.shape
    l = k + p
    if not (k >= 1 and p >= 0 and q >= 0 and l <= min(m, n)):
        raise ValueError("need k >= 1, p >= 0, q >= 0, k + p <= min(m, n)")
    if orth == "householder":
        orthf = orthonormalize
    elif orth == "cholqr2":
        orthf = _cholqr2
    elif orth == "none":
        orthf = lambda Y: Y
    else:
        raise ValueError(orth)

    Omega = sketch(seed, n, l, dtype)                 # step 1
    Y = range_product(A, Omega)                       # step 2, q = 0 part
    Q = orthf(Y)
    for _ in range(q):                                # step 2, power scheme
        Z = orthf(adjoint_product(A, Q))
        Q = orthf(range_product(A, Z))
    if orth == "none":
        Q = orthonormalize(Q)                         # step 3
    B = adjoint_product(A, Q).T                       # step 4: B = Q^T A
    Ub, sig, Vt = small_svd(B)                        # step 5
    U = range_product(Q, Ub[:, :k])                   # step 6
    return SimpleNamespace(S=sig[:k].copy(), U=U, Vt=Vt[:k].copy(),
                           Omega=Omega, Q=Q, B=B, S_all=sig, Ub=Ub, Vt_all=Vt)


def reconstruction_error(A, U, S, Vt, block=4096):
    """||A - U diag(S) Vt||_F accumulated row block by row block in fp64."""
    A = np.asarray(A)
    US = np.asarray(U, dtype=np.float64) * np.asarray(S, dtype=np.float64)
    Vt = np.asarray(Vt, dtype=np.float64)
    acc = 0.0
    for r0 in range(0, A.shape[0], block):
        R = A[r0:r0 + block].astype(np.float64) - US[r0:r0 + block] @ Vt
        acc += float(np.sum(R * R))
    return np.sqrt(acc)
