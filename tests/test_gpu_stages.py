"""GPU parity, stage by stage: every step of Algorithm 1 through the C ABI
against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

import workloads
from oracle import philox as ophilox
from oracle import rsvd as orc
from oracle import jacobi as ojacobi
import parity
from gpu_util import ctx, to_dev, to_np, say

pytestmark = pytest.mark.gpu

NPDT = {"f32": np.float32, "f64": np.float64}
CODE = {"f32": 0, "f64": 1}


# ---------------------------------------------------------------- step 1: sketch
def test_philox_raw_bit_exact():
    c = ctx()
    for seed, first, n in ((0, 0, 1 << 20), (0x0123456789ABCDEF, (1 << 32) - 500, 1000), (7, 12345, 1)):
        say("philox raw", seed, first, n)
        got = to_np(c.rsvd_stage_philox_raw(seed, first, n)).view(np.uint32)
        want = ophilox.philox_groups(seed, first, n)
        assert (got == want).all()
    got = to_np(c.rsvd_stage_philox_raw(3, 10, 64, stream_id=5)).view(np.uint32)
    assert (got == ophilox.philox_groups(3, 10, 64, stream=5)).all()


@pytest.mark.parametrize("dt", ["f32", "f64"])
@pytest.mark.parametrize("shape", [(2000, 80), (1001, 21), (1, 1), (3, 5)])
def test_sketch_matches_oracle(dt, shape):
    say("sketch", dt, shape)
    n, l = shape
    got = to_np(ctx().rsvd_stage_sketch(11, n, l, CODE[dt])).astype(np.float64)
    want = ophilox.philox_normal(11, n, l, NPDT[dt]).astype(np.float64)
    # fp32: both sides round one fp64 value, so they differ by at most one fp32 ulp where the
    # fp64 libm results straddle a rounding boundary.  fp64: log, sqrt, sincos and two
    # multiplications, each within ~1-2 ulp on either side -> 8 eps relative.
    eps = np.finfo(NPDT[dt]).eps
    tol = (1.0 if dt == "f32" else 8.0) * eps * np.maximum(1.0, np.abs(want))
    assert (np.abs(got - want) <= tol).all()
    if dt == "f32":
        assert (got != want).mean() < 1e-3


def test_sketch_strided_and_empty():
    import torch
    c = ctx()
    buf = torch.full((50, 16), -7.0, dtype=torch.float64, device="cuda:0")
    c.rsvd_stage_sketch(2, 50, 10, 1, out=buf[:, :10])
    got = to_np(buf)
    want = ophilox.philox_normal(2, 50, 10, np.float64)
    np.testing.assert_allclose(got[:, :10], want, rtol=1e-14, atol=1e-15)
    assert (got[:, 10:] == -7.0).all()
    assert c.rsvd_stage_sketch(2, 0, 10, 1).shape == (0, 10)


# ---------------------------------------------------------------- steps 2, 4, 6: products
GEMM_CASES = [
    # m, n, l : several tiles with ragged tails, vector and scalar load paths, split-K shapes
    (333, 517, 20), (1000, 260, 80), (130, 4100, 16), (4100, 130, 24), (257, 129, 21),
    (96, 64, 64), (700, 300, 120), (5000, 100, 100), (64, 9000, 48), (513, 515, 7),
]


def _gemm_check(got, A, X, K, dt):
    want = A @ X
    eps = np.finfo(NPDT[dt]).eps
    bound = K * eps * (np.abs(A) @ np.abs(X)) + 1e-300      # rigorous: any summation order
    assert (np.abs(got - want) <= bound).all(), float(np.max(np.abs(got - want) / bound))
    rel = np.linalg.norm(got - want) / np.linalg.norm(want)
    assert rel <= 4 * np.sqrt(K) * eps, rel
    return rel


@pytest.mark.parametrize("dt", ["f32", "f64"])
@pytest.mark.parametrize("m,n,l", GEMM_CASES)
def test_range_product(dt, m, n, l):
    say("gemm_an", dt, m, n, l)
    A = workloads.gaussian_matrix(m, n, 1, NPDT[dt])
    X = workloads.gaussian_matrix(n, l, 2, NPDT[dt])
    got = to_np(ctx().rsvd_stage_gemm_an(to_dev(A), to_dev(X))).astype(np.float64)
    _gemm_check(got, A.astype(np.float64), X.astype(np.float64), n, dt)


@pytest.mark.parametrize("dt", ["f32", "f64"])
@pytest.mark.parametrize("m,n,l", GEMM_CASES)
def test_adjoint_product(dt, m, n, l):
    say("gemm_atn", dt, m, n, l)
    A = workloads.gaussian_matrix(m, n, 3, NPDT[dt])
    X = workloads.gaussian_matrix(m, l, 4, NPDT[dt])
    got = to_np(ctx().rsvd_stage_gemm_atn(to_dev(A), to_dev(X))).astype(np.float64)
    _gemm_check(got, A.astype(np.float64).T, X.astype(np.float64), m, dt)


def test_products_with_leading_dimensions():
    import torch
    A = workloads.gaussian_matrix(300, 200, 5, np.float32)
    X = workloads.gaussian_matrix(200, 40, 6, np.float32)
    Abig = torch.zeros((300, 212), dtype=torch.float32, device="cuda:0")
    Abig[:, :200] = to_dev(A)
    Xbig = torch.zeros((200, 44), dtype=torch.float32, device="cuda:0")
    Xbig[:, :40] = to_dev(X)
    got = to_np(ctx().rsvd_stage_gemm_an(Abig[:, :200], Xbig[:, :40])).astype(np.float64)
    _gemm_check(got, A.astype(np.float64), X.astype(np.float64), 200, "f32")


@pytest.mark.parametrize("dt", ["f32", "f64"])
@pytest.mark.parametrize("m,l,k,tr", [(1000, 80, 64, False), (517, 20, 10, True), (2000, 120, 100, True),
                                      (130, 33, 7, False)])
def test_lift(dt, m, l, k, tr):
    say("lift", dt, m, l, k, tr)
    Q = workloads.gaussian_matrix(m, l, 7, NPDT[dt])
    W = workloads.gaussian_matrix(l, l, 8, NPDT[dt])
    got = to_np(ctx().rsvd_stage_lift(to_dev(Q), to_dev(W), k, transpose_out=tr)).astype(np.float64)
    if tr:
        got = got.T
    _gemm_check(got, Q.astype(np.float64), W.astype(np.float64)[:, :k], l, dt)


# ---------------------------------------------------------------- step 3: orthonormalisation
@pytest.mark.parametrize("dt", ["f32", "f64"])
@pytest.mark.parametrize("rows,l,cond", [(512, 20, 10.0), (3000, 80, 1e3), (1000, 120, 50.0), (129, 33, 5.0),
                                         (10000, 64, 1e2), (2000, 160, 30.0), (3000, 288, 1e2), (5000, 576, 10.0),
                                         (1500, 200, 1e3), (2500, 900, 10.0)])     # 900: past the strip inverse's LDS limit
def test_orth_full_rank_matches_householder(dt, rows, l, cond):
    say("orth", dt, rows, l, cond)
    Y = workloads.graded_matrix(rows, l, cond, seed=20, dtype=NPDT[dt])
    Qg, Rg, info = ctx().rsvd_stage_orth(to_dev(Y), want_r=True)
    Qg, Rg = to_np(Qg).astype(np.float64), to_np(Rg)
    Qo, Ro = orc.qr_positive(Y.astype(np.float64))
    eps = np.finfo(NPDT[dt]).eps
    assert info.refilled_columns == 0 and info.status == 0
    assert parity.orthonormality(Qg) <= 10 * l * eps
    # the positive-diagonal QR is unique; CholeskyQR2 reaches it to ~eps * cond
    assert np.abs(Qg - Qo).max() <= 20 * eps * cond
    assert np.abs(Rg - Ro).max() <= 20 * eps * cond * np.abs(Ro).max()
    assert np.abs(np.tril(Rg, -1)).max() == 0.0


@pytest.mark.parametrize("rows,l,cond", [(2000, 48, 1e9), (1500, 96, 1e11), (3000, 160, 1e10), (800, 20, 1e8),
                                         (4000, 288, 1e9)])
def test_orth_ill_conditioned_fp64_panel_matches_householder(rows, l, cond):
    """fp64 panels whose singular values span far more than the six decades one CholeskyQR round resolves (the
    paper's step 3 is a Householder QR, which keeps every direction down to the rounding level): the raised
    pivots of the first round and the additional round must deliver the same Q and R, with no column replaced."""
    say("orth ill-conditioned", rows, l, cond)
    Y = workloads.graded_matrix(rows, l, cond, seed=21, dtype=np.float64)
    Qg, Rg, info = ctx().rsvd_stage_orth(to_dev(Y), want_r=True)
    Qg, Rg = to_np(Qg), to_np(Rg)
    Qo, Ro = orc.qr_positive(Y)
    eps = np.finfo(np.float64).eps
    say("  raised", info.raised_pivots, "refilled", info.refilled_columns)
    assert info.status == 0 and info.refilled_columns == 0 and info.raised_pivots > 0
    assert parity.orthonormality(Qg) <= 10 * l * eps
    assert np.linalg.norm(Y - Qg @ Rg) <= 50 * l * eps * np.linalg.norm(Y)
    assert np.abs(np.tril(Rg, -1)).max() == 0.0
    # Householder QR itself fixes column j of Q only to eps * (cond of the leading j columns); compare at that level
    assert np.abs(Qg - Qo).max() <= 50 * eps * cond
    assert np.abs(Rg - Ro).max() <= 50 * eps * cond * np.abs(Ro).max()


@pytest.mark.parametrize("dt", ["f32", "f64"])
def test_orth_rank_deficient_input(dt):
    """rank 10 < l = 20 (the situation of the planted rank-10 configuration)."""
    say("orth rank deficient", dt)
    rows, l, r = 512, 20, 10
    B = workloads.gaussian_matrix(rows, r, 30) @ workloads.gaussian_matrix(r, l, 31)
    Y = B.astype(NPDT[dt])
    Qg, Rg, info = ctx().rsvd_stage_orth(to_dev(Y), want_r=True)
    Qg, Rg = to_np(Qg).astype(np.float64), to_np(Rg)
    eps = np.finfo(NPDT[dt]).eps
    say("  refilled", info.refilled_columns)
    assert parity.orthonormality(Qg) <= 10 * l * eps
    Y64 = Y.astype(np.float64)
    # range(Q) contains range(Y), and Y = Q R
    assert np.linalg.norm(Y64 - Qg @ (Qg.T @ Y64)) <= 50 * l * eps * np.linalg.norm(Y64)
    assert np.linalg.norm(Y64 - Qg @ Rg) <= 50 * l * eps * np.linalg.norm(Y64)
    if dt == "f64":
        assert info.refilled_columns == l - r


def test_orth_zero_and_nonfinite_input():
    import torch
    Y = torch.zeros((100, 8), dtype=torch.float64, device="cuda:0")
    Q, _, info = ctx().rsvd_stage_orth(Y)
    assert info.refilled_columns == 8
    assert parity.orthonormality(to_np(Q)) <= 1e-13
    Y = to_dev(workloads.gaussian_matrix(100, 8, 1))
    Y[5, 3] = float("nan")
    from paper_2110_03423_amd import RsvdError
    with pytest.raises(RsvdError) as ei:
        ctx().rsvd_stage_orth(Y)
    assert ei.value.code == 1


# ---------------------------------------------------------------- step 5: small SVD
def _svd_check(sig, X, W, M, dt, name):
    l = M.shape[0]
    tol = parity.jacobi_tol(l, dt)
    want = np.linalg.svd(M, compute_uv=False)
    smax = want[0]
    assert np.abs(sig - want).max() <= tol * smax, (name, np.abs(sig - want).max())
    assert (np.diff(sig) <= 0).all()
    assert np.linalg.norm(W.T @ W - np.eye(l)) <= tol
    nz = sig > 100 * l * np.finfo(NPDT[dt]).eps * smax
    assert np.linalg.norm((X.T @ X)[np.ix_(nz, nz)] - np.eye(nz.sum())) <= tol
    assert np.linalg.norm(X * sig @ W.T - M) <= tol * smax


@pytest.mark.parametrize("dt", ["f32", "f64"])
@pytest.mark.parametrize("l", [2, 5, 20, 33, 64, 80, 96, 128, 129, 160, 200, 288, 333, 576])
def test_jacobi_matches_oracle(dt, l):
    say("jacobi", dt, l)
    M = workloads.gaussian_matrix(l, l, 40 + l, NPDT[dt])
    sig, X, W, info = ctx().rsvd_stage_jacobi(to_dev(M))
    sig, X, W = (to_np(t).astype(np.float64) for t in (sig, X, W))
    say("  sweeps", info.jacobi_sweeps)
    assert info.status == 0 and 1 <= info.jacobi_sweeps <= 20
    M64 = M.astype(np.float64)
    _svd_check(sig, X, W, M64, dt, "gaussian")
    # every column goes through ~l rotations per sweep: their rounding errors must add up like a random walk
    # (a rotation whose c^2 + s^2 is off by a few 1e-8 in the same direction every time shows up here)
    want = np.linalg.svd(M64, compute_uv=False)
    assert np.abs(sig - want).max() <= 20 * np.finfo(NPDT[dt]).eps * np.sqrt(l) * want[0]
    if l <= 33:       # brute-force Jacobi oracle on the small ones: vectors up to sign
        Xo, so, Wo, _ = ojacobi.jacobi_svd(M64)
        tol = 1e3 * np.finfo(NPDT[dt]).eps / np.min(np.abs(np.diff(so)) / so[:-1]) if l > 1 else 1
        assert np.abs(np.abs(np.sum(X * Xo, axis=0)) - 1).max() <= min(0.1, tol)
        assert np.abs(np.abs(np.sum(W * Wo, axis=0)) - 1).max() <= min(0.1, tol)


@pytest.mark.parametrize("dt", ["f32", "f64"])
def test_jacobi_special_matrices(dt):
    say("jacobi special", dt)
    c = ctx()
    T = NPDT[dt]
    eps = np.finfo(T).eps
    d = np.array([3.0, 0.5, 7.0, 1.0, 0.0, 2.0])
    sig, X, W, info = c.rsvd_stage_jacobi(to_dev(np.diag(d).astype(T)))
    np.testing.assert_allclose(to_np(sig), np.sort(d)[::-1], rtol=4 * eps, atol=0)
    assert info.jacobi_sweeps == 1
    Q = workloads.orthonormal_factor(24, 24, 5).astype(T)
    sig, X, W, info = c.rsvd_stage_jacobi(to_dev(Q))
    np.testing.assert_allclose(to_np(sig), np.ones(24), rtol=50 * eps)
    u, v = workloads.gaussian_matrix(16, 1, 1), workloads.gaussian_matrix(16, 1, 2)
    M = (u @ v.T).astype(T)
    sig, X, W, info = c.rsvd_stage_jacobi(to_dev(M))
    sig = to_np(sig).astype(np.float64)
    assert sig[0] == pytest.approx(np.linalg.norm(u) * np.linalg.norm(v), rel=50 * eps)
    assert (sig[1:] <= 50 * eps * sig[0]).all()
    G = workloads.graded_matrix(32, 32, 1e6 if dt == "f64" else 1e3, seed=9, dtype=T)
    sig, X, W, info = c.rsvd_stage_jacobi(to_dev(G))
    _svd_check(*(to_np(t).astype(np.float64) for t in (sig, X, W)), G.astype(np.float64), dt, "graded")


@pytest.mark.parametrize("dt", ["f32", "f64"])
@pytest.mark.parametrize("n,l", [(256, 20), (2000, 80), (1000, 120), (300, 33), (2000, 288), (1000, 160)])
def test_small_svd_of_projected_factor(dt, n, l):
    say("small_svd", dt, n, l)
    Bt = workloads.graded_matrix(n, l, 100.0, seed=50, dtype=NPDT[dt])
    sig, Ub, V, info = ctx().rsvd_stage_small_svd(to_dev(Bt))
    sig, Ub, V = (to_np(t).astype(np.float64) for t in (sig, Ub, V))
    B = Bt.astype(np.float64).T
    Uo, so, Vto = orc.small_svd(B)
    eps = np.finfo(NPDT[dt]).eps
    tol = parity.jacobi_tol(l, dt)
    assert np.abs(sig - so).max() <= tol * so[0]
    assert np.linalg.norm(Ub * sig @ V.T - B) <= tol * so[0]
    assert parity.orthonormality(V) <= tol and parity.orthonormality(Ub) <= tol
    # graded spectrum 1 .. 1/100 in l steps: relative gaps ~ ln(100)/l, vectors well defined
    gap = np.log(100.0) / l
    assert np.abs(np.abs(np.sum(Ub * Uo, axis=0)) - 1).max() <= 100 * l * eps / gap
    assert np.abs(np.abs(np.sum(V * Vto.T, axis=0)) - 1).max() <= 100 * l * eps / gap


HARD_FACTORS = [  # (dtype, n, l, singular values of B): steep decays and flat clusters, orders on both Jacobi paths
    ("f32", 900, 96, lambda i, l: 10.0 ** (-i / 16.0), 12),                      # six decades
    ("f32", 1200, 261, lambda i, l: 10.0 ** (-i / 40.0), 12),                    # six and a half, block path
    ("f64", 800, 60, lambda i, l: 10.0 ** (-i / 5.0), 12),                       # twelve decades
    ("f64", 1000, 200, lambda i, l: 10.0 ** (-i / 20.0), 12),                    # ten, block path
    # flat clusters: inside one the sweeps gain a constant factor only, down to the rounding level of the type
    ("f32", 900, 80, lambda i, l: np.where(i < l // 2, 1.0, 1e-3), 12),
    ("f64", 1100, 200, lambda i, l: np.where(i < l // 2, 1.0, 1e-3), 20),
    ("f64", 700, 120, lambda i, l: np.where(i < l // 4, 10.0 ** (-i / 5.0), 1e-6), 20),   # a steep head above a flat tail
]


@pytest.mark.parametrize("dt,n,l,spec,max_sweeps", HARD_FACTORS,
                         ids=[f"{c[0]}-{c[1]}x{c[2]}-{j}" for j, c in enumerate(HARD_FACTORS)])
def test_small_svd_of_steep_and_clustered_factors(dt, n, l, spec, max_sweeps):
    """B with a steep spectrum or with clusters of equal singular values, in general position (no power iteration
    has lined its rows up): the rotations act on the rows of the triangular factor of B^T, which are graded like
    the singular values, and need about as many sweeps as on an easy factor (on its columns they needed 20 and
    more, or ran into the sweep cap); inside a cluster the vectors come out orthogonal to the rounding level."""
    say("small_svd hard", dt, n, l)
    T = NPDT[dt]
    i = np.arange(l, dtype=np.float64)
    s = np.asarray(spec(i, l), dtype=np.float64) * np.ones(l)
    B = (workloads.orthonormal_factor(l, l, 70) * s) @ workloads.orthonormal_factor(n, l, 71).T
    Bt = np.ascontiguousarray(B.T.astype(T))
    sig, Ub, V, info = ctx().rsvd_stage_small_svd(to_dev(Bt))
    sig, Ub, V = (to_np(t).astype(np.float64) for t in (sig, Ub, V))
    B = Bt.astype(np.float64).T
    so = np.linalg.svd(B, compute_uv=False)
    tol = parity.jacobi_tol(l, dt)
    say("  sweeps", info.jacobi_sweeps)
    assert info.status == 0 and info.jacobi_sweeps <= max_sweeps, info.jacobi_sweeps
    assert np.abs(sig - so).max() <= tol * so[0]
    big = so > so[0] * (1e-5 if dt == "f32" else 1e-10)
    assert (np.abs(sig - so)[big] / so[big]).max() <= (1e-3 if dt == "f32" else 1e-5)
    assert np.linalg.norm(Ub * sig @ V.T - B) <= tol * so[0]
    # singular values at the rounding level of the whole factor count as zero: their columns of Ub are zero
    live = so > 4 * np.finfo(T).eps * np.linalg.norm(so)
    assert parity.orthonormality(V) <= tol and parity.orthonormality(Ub[:, live]) <= tol
    assert all(np.abs(np.linalg.norm(Ub[:, j]) - 1) <= tol or not Ub[:, j].any() for j in np.where(~live)[0])


def test_small_svd_rank_deficient_factor():
    say("small_svd rank deficient")
    n, l, r = 256, 20, 10
    B = (workloads.gaussian_matrix(l, r, 60) @ workloads.gaussian_matrix(r, n, 61))
    sig, Ub, V, info = ctx().rsvd_stage_small_svd(to_dev(np.ascontiguousarray(B.T)))
    sig, Ub, V = (to_np(t) for t in (sig, Ub, V))
    so = np.linalg.svd(B, compute_uv=False)
    np.testing.assert_allclose(sig[:r], so[:r], rtol=1e-11)
    assert (sig[r:] <= 1e-12 * so[0]).all()
    assert np.linalg.norm(Ub[:, :r] * sig[:r] @ V[:, :r].T - B) <= 1e-12 * so[0]


def test_argument_errors_are_reported():
    import torch
    from paper_2110_03423_amd import RsvdError
    c = ctx()
    A = torch.zeros((10, 6), dtype=torch.float64, device="cuda:0")
    for k, p, q in ((0, 2, 1), (3, -1, 1), (3, 2, -1), (5, 2, 0)):
        with pytest.raises(RsvdError) as ei:
            c.rsvd_run(A, k, p, q, workspace=torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0"))
        assert ei.value.code < 0
    with pytest.raises(RsvdError) as ei:
        c.rsvd_run(A, 2, 2, 1, workspace=torch.zeros(256, dtype=torch.uint8, device="cuda:0"))
    assert ei.value.code == -19
