"""Pins for the brute-force Jacobi SVD and, through it, for the LAPACK call
the oracle uses in step 5 of Algorithm 1."""
import numpy as np
import pytest

from oracle import jacobi, rsvd
import workloads


def test_diagonal_matrix():
    d = np.array([3.0, 0.5, 7.0, 1.0])
    X, s, W, _ = jacobi.jacobi_svd(np.diag(d))
    np.testing.assert_allclose(s, [7.0, 3.0, 1.0, 0.5], rtol=1e-15)
    np.testing.assert_allclose(np.abs(X), np.eye(4)[:, [2, 0, 3, 1]], atol=1e-15)


def test_rank_one_outer_product():
    u = np.array([1.0, 2.0, -2.0, 4.0, 0.0])
    v = np.array([3.0, -4.0, 12.0])
    X, s, W, _ = jacobi.jacobi_svd(np.outer(u, v))
    assert s[0] == pytest.approx(5.0 * 13.0, rel=1e-14)
    assert np.all(s[1:] < 1e-13)
    assert abs(X[:, 0] @ u) / 5.0 == pytest.approx(1.0, rel=1e-14)
    assert abs(W[:, 0] @ v) / 13.0 == pytest.approx(1.0, rel=1e-14)


def test_orthogonal_matrix_has_unit_singular_values():
    Q = workloads.orthonormal_factor(12, 12, 5)
    X, s, W, sweeps = jacobi.jacobi_svd(Q)
    np.testing.assert_allclose(s, np.ones(12), rtol=1e-14)
    assert sweeps == 1


def test_two_by_two_closed_form():
    a, b, c, d = 1.5, -0.25, 2.0, 0.75
    M = np.array([[a, b], [c, d]])
    # singular values of a 2x2 matrix from its Frobenius norm and determinant
    f2, det = a * a + b * b + c * c + d * d, abs(a * d - b * c)
    s1 = np.sqrt((f2 + np.sqrt(f2 * f2 - 4 * det * det)) / 2)
    s2 = det / s1
    X, s, W, _ = jacobi.jacobi_svd(M)
    np.testing.assert_allclose(s, [s1, s2], rtol=1e-14)
    np.testing.assert_allclose(X * s @ W.T, M, atol=1e-15)


@pytest.mark.parametrize("shape,seed", [((7, 7), 0), ((33, 20), 1), ((64, 64), 2), ((40, 1), 3)])
def test_lapack_step_matches_brute_force(shape, seed):
    M = workloads.gaussian_matrix(*shape, seed=seed)
    X, s, W, sweeps = jacobi.jacobi_svd(M)
    U, sl, Vt = rsvd.small_svd(M)
    np.testing.assert_allclose(s, sl, rtol=1e-12)
    np.testing.assert_allclose(X * s @ W.T, M, atol=1e-12)
    np.testing.assert_allclose(np.abs(np.sum(U * X, axis=0)), 1.0, atol=1e-9)
    np.testing.assert_allclose(np.abs(np.sum(Vt.T * W, axis=0)), 1.0, atol=1e-9)
    assert np.linalg.norm(W.T @ W - np.eye(shape[1])) < 1e-13
    assert sweeps <= 12          # quadratic convergence: a handful of sweeps


def test_graded_and_singular_inputs():
    M = workloads.graded_matrix(48, 24, 1e10, seed=4)
    X, s, W, _ = jacobi.jacobi_svd(M)
    want = 1e10 ** (-np.arange(24) / 23)
    np.testing.assert_allclose(s, want, rtol=1e-5)       # limit set by how M was built (abs error eps*s_max)
    np.testing.assert_allclose(s, np.linalg.svd(M, compute_uv=False), rtol=1e-5)
    Z = np.zeros((10, 4))
    Z[:, 1] = 2.0
    X, s, W, _ = jacobi.jacobi_svd(Z)
    np.testing.assert_allclose(s, [2.0 * np.sqrt(10), 0, 0, 0], atol=1e-15)
