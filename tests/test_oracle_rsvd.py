"""Pins for the oracle's Algorithm 1 (the whole randomized k-SVD) against what
the mathematics fixes: exact recovery when rank(A) <= l, reduction to a full
SVD when l = min(m, n), the Eckart-Young lower bound, the range finder's
expectation bound, Ritz values below the true singular values, and
invariance under the re-orthonormalisation schedule."""
import numpy as np
import pytest

from oracle import rsvd as orc
import workloads
from workloads import CONFIGS, scaled
import parity


@pytest.fixture(scope="module")
def cfg1():
    cfg = CONFIGS[1]
    return cfg, workloads.build(cfg)


def test_orthonormalize_invariants():
    Y = workloads.graded_matrix(300, 24, 1e6, seed=11)
    Q = orc.orthonormalize(Y)
    eps = np.finfo(np.float64).eps
    assert parity.orthonormality(Q) <= 10 * 24 * eps
    assert np.linalg.norm(Y - Q @ (Q.T @ Y)) <= 10 * 24 * eps * np.linalg.norm(Y)
    Qp, R = orc.qr_positive(Y)
    assert (np.diag(R) >= 0).all() and np.allclose(np.tril(R, -1), 0)
    np.testing.assert_allclose(Qp @ R, Y, atol=1e-14)


def test_products_are_plain_products():
    A = workloads.gaussian_matrix(9, 5, seed=1)
    X = workloads.gaussian_matrix(5, 3, seed=2)
    W = workloads.gaussian_matrix(9, 3, seed=3)
    want = np.array([[sum(A[i, t] * X[t, j] for t in range(5)) for j in range(3)] for i in range(9)])
    np.testing.assert_allclose(orc.range_product(A, X), want, rtol=1e-14)
    want_t = np.array([[sum(A[t, i] * W[t, j] for t in range(9)) for j in range(3)] for i in range(5)])
    np.testing.assert_allclose(orc.adjoint_product(A, W), want_t, rtol=1e-14)


def test_config1_exact_recovery(cfg1):
    """rank(A) = 10 <= l = 20: the output is the exact compact SVD, truncated to k."""
    cfg, A = cfg1
    out = orc.rsvd(A, cfg.k, cfg.p, cfg.q, cfg.seed, cfg.np_dtype)
    want = 10.0 ** (-np.arange(10) / 5.0)
    np.testing.assert_allclose(out.S, want, rtol=1e-12)
    U = workloads.orthonormal_factor(cfg.m, cfg.rank, 1000 + cfg.cid)
    V = workloads.orthonormal_factor(cfg.n, cfg.rank, 2000 + cfg.cid)
    np.testing.assert_allclose(np.abs(np.sum(out.U * U, axis=0)), 1.0, atol=1e-11)
    np.testing.assert_allclose(np.abs(np.sum(out.Vt.T * V, axis=0)), 1.0, atol=1e-11)
    # signs of u_i and v_i are consistent: the product reproduces A
    assert orc.reconstruction_error(A, out.U, out.S, out.Vt) <= 1e-13 * np.linalg.norm(A)
    assert out.U.shape == (cfg.m, cfg.k) and out.Vt.shape == (cfg.k, cfg.n)
    assert out.Omega.shape == (cfg.n, cfg.l) and out.B.shape == (cfg.l, cfg.n)
    assert (out.S_all[10:] <= 1e-13).all()


@pytest.mark.parametrize("q", [0, 1, 3])
def test_exact_recovery_any_q_and_wide_input(q):
    cfg = scaled(CONFIGS[1], 96, 160, rank=7, k=7, p=3)      # m < n as well
    A = workloads.build(cfg)
    out = orc.rsvd(A, cfg.k, cfg.p, q, seed=3, dtype=np.float64)
    np.testing.assert_allclose(out.S, 10.0 ** (-np.arange(7) / 5.0), rtol=1e-11)
    assert orc.reconstruction_error(A, out.U, out.S, out.Vt) <= 1e-12 * np.linalg.norm(A)


def test_full_sketch_reduces_to_svd():
    A = workloads.gaussian_matrix(40, 12, seed=21)
    out = orc.rsvd(A, 5, 7, 1, seed=0, dtype=np.float64)      # l = 12 = min(m, n)
    U, s, Vt = np.linalg.svd(A, full_matrices=False)
    np.testing.assert_allclose(out.S, s[:5], rtol=1e-12)
    np.testing.assert_allclose(np.abs(np.sum(out.U * U[:, :5], axis=0)), 1.0, atol=1e-10)
    np.testing.assert_allclose(np.abs(np.sum(out.Vt * Vt[:5], axis=1)), 1.0, atol=1e-10)


@pytest.fixture(scope="module")
def decay_case():
    """1/8-scale replica of config 2 (exponentially decaying full-rank spectrum)."""
    cfg = scaled(CONFIGS[2], 1250, 250, k=16, p=24)
    return cfg, workloads.build(cfg).astype(np.float64), cfg.singular_values()


def test_eckart_young_and_range_finder_bounds(decay_case):
    cfg, A, s = decay_case
    k, p = cfg.k, cfg.p
    tail = np.sqrt(np.sum(s[k:] ** 2))
    errs = []
    for q in (0, 1, 2):
        e = []
        for seed in range(8):
            out = orc.rsvd(A, k, p, q, seed, np.float32)
            err = orc.reconstruction_error(A, out.U, out.S, out.Vt)
            assert err >= tail * (1 - 1e-6)                  # no rank-k matrix does better
            e.append(err)
        errs.append(np.mean(e))
    # expectation bound of the Gaussian range finder (q = 0), tested loosely per draw
    bound = np.sqrt(1 + k / (p - 1)) * tail
    assert errs[0] <= 3 * bound
    # power iterations never hurt on average and approach the optimum
    assert errs[1] <= errs[0] * (1 + 1e-9) and errs[2] <= errs[1] * (1 + 1e-9)
    assert errs[2] <= 1.001 * tail


def test_ritz_values_below_true_and_closed_form_spectrum(decay_case):
    cfg, A, s = decay_case
    true = np.linalg.svd(A, compute_uv=False)
    out = orc.rsvd(A, cfg.k, cfg.p, cfg.q, cfg.seed, np.float32)
    assert (out.S_all <= true[:cfg.l] * (1 + 1e-12)).all()
    # fp32 storage of A perturbs the planted 0.9^i by ~eps32 relative to s_0
    np.testing.assert_allclose(out.S, s[:cfg.k], rtol=1e-5)
    np.testing.assert_allclose(out.S, true[:cfg.k], rtol=1e-7)


def test_schedule_invariance():
    """In exact arithmetic the result depends only on range((A A^T)^q A Omega)."""
    A = workloads.graded_matrix(120, 60, 30.0, seed=31)
    ref = orc.rsvd(A, 8, 6, 2, seed=4, dtype=np.float64)
    for sched in ("cholqr2", "none"):
        alt = orc.rsvd(A, 8, 6, 2, seed=4, dtype=np.float64, orth=sched)
        np.testing.assert_allclose(alt.S_all, ref.S_all, rtol=1e-9)
        assert parity.sin_theta(alt.Q, ref.Q) <= 1e-8
        assert parity.sin_theta(alt.U, ref.U) <= 1e-8
        assert parity.sin_theta(alt.Vt.T, ref.Vt.T) <= 1e-8


def test_sketch_is_the_philox_stream_rounded_to_dtype():
    from oracle import philox
    Om = orc.sketch(7, 50, 12, np.float32)
    assert Om.dtype == np.float64
    assert (Om == philox.philox_normal(7, 50, 12, np.float32).astype(np.float64)).all()
    assert (Om.astype(np.float32).astype(np.float64) == Om).all()


def test_argument_checks():
    A = np.zeros((10, 6))
    for k, p, q in ((0, 2, 1), (3, -1, 1), (3, 2, -1), (5, 2, 0)):
        with pytest.raises(ValueError):
            orc.rsvd(A, k, p, q, 0, np.float64)


def test_parity_metric_helpers():
    sig = np.array([10.0, 5.0, 4.9999, 4.9998, 1.0, 0.5])
    assert parity.clusters(sig, 1e-4, 4) == [(0, 1), (1, 4)]
    assert parity.clusters(sig, 1e-4, 3) == [(0, 1), (1, 4)]        # run straddles k = 3
    Q = workloads.orthonormal_factor(30, 4, 1)
    assert parity.sin_theta(Q, Q @ workloads.orthonormal_factor(4, 4, 2)) < 1e-14
    P = workloads.orthonormal_factor(30, 30, 3)
    assert parity.sin_theta(P[:, :4], P[:, 4:8]) == pytest.approx(1.0)


def test_paper_fast_decay_accuracy_claim():
    """Experiments, performance comparison: on the fast-decay spectrum the randomized values can be held within
    1e-8 (relative) of a full SVD; how many power iterations that takes follows (sigma_l / sigma_i)^(4q+2)."""
    cfg = workloads.paper_case("fast", 300, 0.05, m=600)
    A = workloads.build(cfg)
    true = np.linalg.svd(A, compute_uv=False)[:cfg.k]
    np.testing.assert_allclose(true, workloads.PAPER_SPECTRA["fast"](np.arange(cfg.k)), rtol=1e-10)
    worst = []
    for q in (1, 2, 4):
        out = orc.rsvd(A, cfg.k, 10, q, 0, np.float64)
        worst.append(np.max(np.abs(out.S - true) / true))
    assert worst[0] > worst[1] > worst[2] and worst[2] <= 1e-8       # q = 4, p = 10 reaches the paper's level
    out = orc.rsvd(A, cfg.k, 30, 2, 0, np.float64)                    # so does q = 2 with more oversampling
    assert np.max(np.abs(out.S - true) / true) <= 1e-8
