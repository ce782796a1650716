"""GPU parity of the whole randomized k-SVD (Algorithm 1) through rsvd_run
against the CPU oracle, at reduced and at full benchmark sizes."""
import dataclasses

import numpy as np
import pytest

import workloads
from workloads import CONFIGS, scaled
from oracle import rsvd as orc
import parity
from gpu_util import ctx, to_dev, to_np, say

pytestmark = pytest.mark.gpu


def run_and_compare(cfg, A_dev, A_host, q=None, note=""):
    """Run the HIP path and the oracle on the same A; assert the benchmark spec's tolerances."""
    import torch
    q = cfg.q if q is None else q
    k, p, l, dt = cfg.k, cfg.p, cfg.l, cfg.dtype
    m, n = cfg.m, cfg.n
    c = ctx()
    say(f"rsvd {cfg.name} {dt} k={k} p={p} q={q} {note}")
    S, U, Vt, info = c.rsvd_run(A_dev, k, p, q, seed=cfg.seed)
    Sa, Ua, Vta, _ = c.rsvd_run(A_dev, l, 0, q, seed=cfg.seed)          # same sketch, no truncation
    torch.cuda.synchronize()
    S, U, Vt, Sa, Ua, Vta = (to_np(t).astype(np.float64) for t in (S, U, Vt, Sa, Ua, Vta))
    say(f"  info: status={info.status} sweeps={info.jacobi_sweeps} refilled={info.refilled_columns}")
    assert info.status == 0
    assert (S == Sa[:k]).all() and (U == Ua[:, :k]).all()               # deterministic

    o = orc.rsvd(A_host, k, p, q, cfg.seed, cfg.np_dtype)
    res = parity.check_triplets(S, U, Vt, o.S, o.U, o.Vt, dt, m, n,
                                S_all_o=o.S_all, U_all_o=o.Q @ o.Ub, Vt_all_o=o.Vt_all,
                                S_all_g=Sa, U_all_g=Ua, Vt_all_g=Vta)
    eps = parity.EPS[dt]
    sig = parity.significant(o.S, dt, m, n)
    ns = int(sig.sum())
    assert parity.orthonormality(U[:, :ns]) <= parity.jacobi_tol(l, dt)
    assert parity.orthonormality(Vt[:ns].T) <= parity.jacobi_tol(l, dt)
    err_g = orc.reconstruction_error(A_host, U, S, Vt)
    err_o = orc.reconstruction_error(A_host, o.U, o.S, o.Vt)
    normA = float(np.sqrt(np.sum(A_host.astype(np.float64) ** 2)))
    say(f"  sv_rel={res['sv_rel_max']:.2e} sinU={res['sin_u']:.2e} sinV={res['sin_v']:.2e} "
        f"clusters={res['clusters']} skipped={res['skipped']} err_g/err_o={err_g / max(err_o, 1e-300):.6f}")
    assert err_g <= 1.01 * err_o + 50 * eps * normA
    # whole-basis angle: the l-dimensional ranges agree
    if ns == l:
        assert parity.sin_theta(Ua, o.Q @ o.Ub) <= parity.ANGLE_TOL[dt]
    return res


SMALL = [
    scaled(CONFIGS[1], 96, 160, rank=7, k=7, p=3),            # wide, exact recovery
    scaled(CONFIGS[1], 200, 200, rank=12, k=10, p=6),
    scaled(CONFIGS[2], 1250, 250, k=16, p=24),
    scaled(CONFIGS[2], 777, 333, k=20, p=13),                  # odd l: scalar load paths
    scaled(CONFIGS[3], 6250, 250, rank=25, k=25, p=5),
    scaled(CONFIGS[4], 1250, 1250, rank=128, k=16, p=4),
    scaled(CONFIGS[5], 2048, 512, rank=16, k=16, p=16),
    scaled(CONFIGS[4], 2500, 2500, rank=512, k=256, p=32),   # l = 288: blocked Cholesky, block Jacobi (fp64)
    scaled(CONFIGS[5], 4096, 2048, rank=512, k=512, p=64),   # l = 576: the same in fp32
    scaled(CONFIGS[3], 3000, 400, rank=50, k=120, p=40),     # l = 160, noise-dominated tail
]


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: c.name)
def test_reduced_configs(cfg):
    A = workloads.build(cfg)
    run_and_compare(cfg, to_dev(A), A)


STEEP = [  # fp64, noise-free spectra that run far below 1e-6 sigma_1 inside the sketch
    (scaled(CONFIGS[1], 936, 2582, rank=41, k=41, p=17), 1),     # 10^(-i/5) to 1e-8, rank < l
    (scaled(CONFIGS[1], 298, 819, rank=84, k=103, p=36), 1),     # ... to the rounding level, l = 139 (blocked kernels)
    (scaled(CONFIGS[1], 600, 400, rank=60, k=40, p=8), 2),       # full-rank sketch, 1e-9.4 at index 47
    (scaled(CONFIGS[1], 1200, 500, rank=50, k=48, p=12), 0),     # no power iteration
    (dataclasses.replace(scaled(CONFIGS[2], 3000, 700, k=120, p=40), dtype="f64"), 2),   # 0.9^i, l = 160: 5e-8 at the end
]


@pytest.mark.parametrize("cfg,q", STEEP, ids=lambda v: v.name if hasattr(v, "name") else f"q{v}")
def test_steep_spectra_in_fp64(cfg, q):
    """Directions between ~1e-6 sigma_1 (what one CholeskyQR round with an fp64 Gram matrix resolves) and the
    rounding level must survive the orthonormalisations, as they do with the Householder QR of the paper's step 3:
    every singular value above 2.2e-10 sigma_1 is held to 1e-5 against the oracle."""
    A = workloads.build(cfg)
    run_and_compare(cfg, to_dev(A), A, q=q)
    _, _, _, info = ctx().rsvd_run(to_dev(A), cfg.k, cfg.p, q, seed=cfg.seed)
    say(f"  raised={info.raised_pivots} refilled={info.refilled_columns}")
    assert info.raised_pivots > 0
    if cfg.rank >= cfg.l and cfg.spectrum(np.float64(cfg.l)) > 1e-10:
        assert info.refilled_columns == 0                  # a full-rank sketch loses no column


GENERAL_POSITION = [  # no power iteration and a steep spectrum: the factor of step 5 is nowhere near diagonal
    (dataclasses.replace(scaled(CONFIGS[2], 1500, 1200, k=200, p=61), spectrum=lambda i: 10.0 ** (-i / 40.0),
                         name="f32-steep-l261"), 12),
    (dataclasses.replace(scaled(CONFIGS[2], 1800, 900, k=160, p=40), dtype="f64", spectrum=lambda i: 10.0 ** (-i / 20.0),
                         name="f64-steep-l200"), 14),
    (dataclasses.replace(scaled(CONFIGS[2], 900, 700, k=70, p=26), spectrum=lambda i: 10.0 ** (-i / 16.0),
                         name="f32-steep-l96"), 10),
]


@pytest.mark.parametrize("cfg,max_sweeps", GENERAL_POSITION, ids=lambda v: v.name if hasattr(v, "name") else f"s{v}")
def test_no_power_iteration_on_steep_spectra(cfg, max_sweeps):
    """q = 0 on spectra that fall by six to ten decades inside the sketch: the small SVD gets a triangular factor in
    general position.  Rotating its columns took 20 and more sweeps or ended in RSVD_ERR_NO_CONVERGENCE; its rows,
    graded like the singular values, converge in about as many sweeps as an easy factor."""
    A = workloads.build(cfg)
    run_and_compare(cfg, to_dev(A), A, q=0)
    _, _, _, info = ctx().rsvd_run(to_dev(A), cfg.k, cfg.p, 0, seed=cfg.seed)
    say(f"  sweeps={info.jacobi_sweeps}")
    assert info.status == 0 and info.jacobi_sweeps <= max_sweeps


@pytest.mark.parametrize("q", [0, 1, 3])
def test_power_iteration_counts(q):
    cfg = scaled(CONFIGS[2], 900, 300, k=12, p=12)
    A = workloads.build(cfg)
    run_and_compare(cfg, to_dev(A), A, q=q)


def test_jobs_and_leading_dimensions():
    import torch
    from paper_2110_03423_amd import JOB_S, JOB_SV
    cfg = scaled(CONFIGS[4], 400, 300, rank=64, k=8, p=8)
    A = workloads.build(cfg)
    c = ctx()
    Abig = torch.zeros((400, 308), dtype=torch.float64, device="cuda:0")
    Abig[:, :300] = to_dev(A)
    S0, U0, Vt0, _ = c.rsvd_run(to_dev(A), cfg.k, cfg.p, cfg.q)
    S1, U1, Vt1, _ = c.rsvd_run(Abig[:, :300], cfg.k, cfg.p, cfg.q)
    assert torch.equal(S0, S1) and torch.equal(U0, U1) and torch.equal(Vt0, Vt1)
    S2, U2, Vt2, _ = c.rsvd_run(to_dev(A), cfg.k, cfg.p, cfg.q, job=JOB_S)
    assert U2 is None and Vt2 is None and torch.equal(S0, S2)
    S3, U3, Vt3, _ = c.rsvd_run(to_dev(A), cfg.k, cfg.p, cfg.q, job=JOB_SV)
    assert U3 is None and torch.equal(Vt0, Vt3)
    # outputs with their own leading dimensions
    Ub = torch.full((400, 12), 9.0, dtype=torch.float64, device="cuda:0")
    Vb = torch.full((cfg.k, 310), 9.0, dtype=torch.float64, device="cuda:0")
    Sb = torch.empty(cfg.k, dtype=torch.float64, device="cuda:0")
    c.rsvd_run(to_dev(A), cfg.k, cfg.p, cfg.q, out=(Sb, Ub[:, :cfg.k], Vb[:, :300]))
    assert torch.equal(Ub[:, :cfg.k], U0) and torch.equal(Vb[:, :300], Vt0)
    assert (Ub[:, cfg.k:] == 9.0).all() and (Vb[:, 300:] == 9.0).all()


def test_seed_changes_the_sketch_not_the_answer():
    cfg = scaled(CONFIGS[1], 300, 200, rank=9, k=9, p=5)
    A = workloads.build(cfg)
    c = ctx()
    S0, _, _, _ = c.rsvd_run(to_dev(A), cfg.k, cfg.p, cfg.q, seed=0)
    S1, _, _, _ = c.rsvd_run(to_dev(A), cfg.k, cfg.p, cfg.q, seed=12345)
    np.testing.assert_allclose(to_np(S0), to_np(S1), rtol=1e-11)
    np.testing.assert_allclose(to_np(S0), 10.0 ** (-np.arange(9) / 5.0), rtol=1e-11)


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_full_size_configs(cid):
    """The benchmark's configurations at full size, oracle run in full beside the HIP path."""
    cfg = CONFIGS[cid]
    A_dev = workloads.build(cfg, device="cuda:0")
    A = to_np(A_dev)
    res = run_and_compare(cfg, A_dev, A, note="(full size)")
    if cid == 1:      # planted spectrum, exact recovery expected
        S, _, _, _ = ctx().rsvd_run(A_dev, cfg.k, cfg.p, cfg.q, seed=cfg.seed)
        np.testing.assert_allclose(to_np(S), 10.0 ** (-np.arange(10) / 5.0), rtol=1e-11)


@pytest.mark.parametrize("m,n,k,p", [(40, 12, 5, 7), (12, 40, 12, 0), (3, 5, 1, 0), (5, 3, 2, 1), (1, 1, 1, 0),
                                     (17, 17, 17, 0), (2, 64, 1, 1)])
@pytest.mark.parametrize("dt", ["f32", "f64"])
def test_tiny_and_full_sketch_shapes(m, n, k, p, dt):
    """Degenerate sizes; with l = min(m, n) the result is the plain SVD (no approximation left)."""
    say("tiny", m, n, k, p, dt)
    npdt = np.float32 if dt == "f32" else np.float64
    A = workloads.gaussian_matrix(m, n, seed=m * 100 + n, dtype=npdt)
    S, U, Vt, info = ctx().rsvd_run(to_dev(A), k, p, 1, seed=3)
    S, U, Vt = (to_np(t).astype(np.float64) for t in (S, U, Vt))
    assert info.status == 0
    A64 = A.astype(np.float64)
    o = orc.rsvd(A64, k, p, 1, 3, npdt)
    eps = parity.EPS[dt]
    np.testing.assert_allclose(S, o.S, rtol=parity.SV_RTOL[dt], atol=10 * eps * o.S[0])
    if k + p == min(m, n):
        np.testing.assert_allclose(S, np.linalg.svd(A64, compute_uv=False)[:k], rtol=parity.SV_RTOL[dt],
                                   atol=10 * eps * o.S[0])
    err_g = orc.reconstruction_error(A64, U, S, Vt)
    err_o = orc.reconstruction_error(A64, o.U, o.S, o.Vt)
    assert err_g <= 1.01 * err_o + 50 * eps * np.linalg.norm(A64)


def test_unaligned_views():
    """Base pointers and leading dimensions that defeat the 16-byte load path."""
    import torch
    cfg = scaled(CONFIGS[2], 301, 203, k=9, p=6)
    A = workloads.build(cfg)
    big = torch.zeros((302, 207), dtype=torch.float32, device="cuda:0")
    view = big[1:, 3:206]                     # offset by 3 floats, ld 207
    view.copy_(to_dev(A))
    c = ctx()
    S0, U0, Vt0, _ = c.rsvd_run(to_dev(A), cfg.k, cfg.p, cfg.q)
    S1, U1, Vt1, _ = c.rsvd_run(view, cfg.k, cfg.p, cfg.q)
    np.testing.assert_allclose(to_np(S1), to_np(S0), rtol=1e-5)
    assert parity.sin_theta(to_np(U1), to_np(U0)) <= 1e-3
    run_and_compare(cfg, view, A)


@pytest.mark.parametrize("kind,n,frac,q", [("fast", 400, 0.05, 2), ("fast", 1000, 0.03, 2), ("sharp", 400, 0.10, 2),
                                          ("sharp", 800, 0.05, 1), ("slow", 400, 0.05, 2), ("slow", 600, 0.10, 3)])
@pytest.mark.parametrize("dt", ["f32", "f64"])
def test_paper_spectra(kind, n, frac, q, dt):
    """The three spectra of the paper's performance comparison (fast 1/i^2, sharp sigmoid, slow 1/i^0.1)
    on A^{2000 x n}, k a percentage of n."""
    cfg = workloads.paper_case(kind, n, frac, dtype=dt, q=q)
    A = workloads.build(cfg)
    run_and_compare(cfg, to_dev(A), A)
    if kind == "fast" and dt == "f64":
        # the paper keeps the relative error against a full SVD at 1e-8 on this kind of input; the error
        # falls like (sigma_l / sigma_k)^(4q+2), so with p = 10 a few more power iterations get there
        S, _, _, _ = ctx().rsvd_run(to_dev(A), cfg.k, cfg.p, 8)
        true = np.linalg.svd(A, compute_uv=False)[:cfg.k]
        assert np.max(np.abs(to_np(S) - true) / true) <= 1e-8


@pytest.mark.parametrize("dt,m,n,k,p,q", [("f64", 600, 200, 12, 8, 2), ("f32", 5000, 300, 20, 10, 2),
                                         ("f32", 3001, 129, 9, 4, 1)])
def test_centered_variant_is_pca(dt, m, n, k, p, q):
    """rsvd_run_centered(A) equals Algorithm 1 on A minus its column means (the paper's PCA application)."""
    say("centered", dt, m, n, k, p, q)
    npdt = np.float32 if dt == "f32" else np.float64
    cfg = scaled(CONFIGS[3], m, n, rank=min(40, n), k=k, p=p)
    base = workloads.build(cfg).astype(np.float64)                    # centred low-rank-plus-noise data
    offs = workloads.gaussian_matrix(1, n, seed=77)                   # feature means of the same size as the data
    A = (base * 0.05 + offs).astype(npdt)
    S, U, Vt, info, mean = ctx().rsvd_run_centered(to_dev(A), k, p, q, seed=cfg.seed)
    S, U, Vt, mean = (to_np(t).astype(np.float64) for t in (S, U, Vt, mean))
    A64 = A.astype(np.float64)
    mu = A64.mean(axis=0)
    eps = parity.EPS[dt]
    assert np.abs(mean - mu).max() <= (2 * eps + 1e-15 * np.sqrt(m)) * np.abs(A64).max()   # fp64 sum, one rounding to dtype
    Ac = A64 - mu
    o = orc.rsvd(Ac, k, p, q, cfg.seed, npdt)
    res = parity.check_triplets(S, U, Vt, o.S, o.U, o.Vt, dt, m, n)
    err_g = orc.reconstruction_error(Ac, U, S, Vt)
    err_o = orc.reconstruction_error(Ac, o.U, o.S, o.Vt)
    say(f"  sv_rel={res['sv_rel_max']:.2e} sinU={res['sin_u']:.2e} sinV={res['sin_v']:.2e} err ratio {err_g / err_o:.6f}")
    assert err_g <= 1.01 * err_o + 50 * eps * np.linalg.norm(Ac)
    # left vectors of a centred matrix are orthogonal to the ones vector
    assert np.abs(U.sum(axis=0)).max() <= 200 * np.sqrt(m) * eps * max(1.0, np.abs(mu).max() / S[-1] * np.sqrt(n))


@pytest.mark.parametrize("dt,m,n,k,p,q,scale", [("f32", 2479, 1668, 60, 4, 2, 1e3), ("f32", 690, 2360, 23, 14, 0, 3e3),
                                               ("f64", 1200, 700, 30, 10, 1, 1e6)])
def test_centered_variant_with_dominant_means(dt, m, n, k, p, q, scale):
    """Feature means `scale` times larger than the spread of the data: the result must be as good as Algorithm 1
    on the explicitly centred matrix, i.e. carry rounding errors of the size of the centred entries (a product
    corrected by a rank-one term after the fact would carry those of the means)."""
    say("centered, dominant means", dt, m, n, k, p, q, scale)
    npdt = np.float32 if dt == "f32" else np.float64
    cfg = scaled(CONFIGS[3], m, n, rank=min(40, n), k=k, p=p)
    base = workloads.build(cfg).astype(np.float64)
    offs = workloads.gaussian_matrix(1, n, seed=78)
    A = (base * 0.05 + scale * 0.05 * offs).astype(npdt)
    S, U, Vt, info, mean = ctx().rsvd_run_centered(to_dev(A), k, p, q, seed=cfg.seed)
    S, U, Vt, mean = (to_np(t).astype(np.float64) for t in (S, U, Vt, mean))
    A64 = A.astype(np.float64)
    Ac = A64 - A64.mean(axis=0)
    assert np.linalg.norm(A64) >= 0.2 * scale * np.linalg.norm(Ac)
    o = orc.rsvd(Ac, k, p, q, cfg.seed, npdt)
    res = parity.check_triplets(S, U, Vt, o.S, o.U, o.Vt, dt, m, n)
    eps = parity.EPS[dt]
    err_g = orc.reconstruction_error(Ac, U, S, Vt)
    err_o = orc.reconstruction_error(Ac, o.U, o.S, o.Vt)
    say(f"  sv_rel={res['sv_rel_max']:.2e} sinU={res['sin_u']:.2e} sinV={res['sin_v']:.2e} err ratio {err_g / err_o:.6f}")
    assert err_g <= 1.01 * err_o + 50 * eps * np.linalg.norm(Ac)


@pytest.mark.parametrize("m,n,k,p", [(800, 300, 20, 10), (900, 500, 150, 10)])     # LDS-resident and block Jacobi
@pytest.mark.parametrize("e", [40, -40])
def test_input_scale_does_not_matter_in_fp32(m, n, k, p, e):
    """A scaled by 2^e (exactly): singular values scale by 2^e, vectors stay.  Products of two squared column
    norms of the small factor leave the fp32 range at these scales (sigma^4 ~ 1e+-54); the Jacobi kernels must
    not form them."""
    say("scale", m, n, k, p, e)
    cfg = scaled(CONFIGS[2], m, n, k=k, p=p)
    A = workloads.build(cfg)
    S0, U0, Vt0, info0 = ctx().rsvd_run(to_dev(A), k, p, 1, seed=3)
    S1, U1, Vt1, info1 = ctx().rsvd_run(to_dev(np.ldexp(A, e).astype(np.float32)), k, p, 1, seed=3)
    assert info0.status == 0 and info1.status == 0
    assert info1.jacobi_sweeps == info0.jacobi_sweeps
    S0, U0, Vt0, S1, U1, Vt1 = (to_np(t).astype(np.float64) for t in (S0, U0, Vt0, S1, U1, Vt1))
    np.testing.assert_allclose(np.ldexp(S1, -e), S0, rtol=1e-5)
    ns = int(parity.significant(S0, "f32", m, n).sum())
    assert parity.orthonormality(U1[:, :ns]) <= parity.jacobi_tol(k + p, "f32")
    assert parity.orthonormality(Vt1[:ns].T) <= parity.jacobi_tol(k + p, "f32")
    assert np.abs(np.abs(np.sum(U0[:, :5] * U1[:, :5], axis=0)) - 1).max() <= 1e-3


@pytest.mark.parametrize("m,n,q,expect", [
    (6000, 300, 3, 1),      # tall, q = 3: the m-side factorisations inside the power scheme are dropped
    (300, 6000, 2, 1),      # wide: the n-side ones
    (2000, 500, 1, 1),      # q = 1: only an n-side one exists
    (2000, 500, 0, 0),      # no power scheme, nothing to drop
])
def test_adaptive_reorthonormalisation(m, n, q, expect):
    """Flat spectrum above a noise floor: the first panel is well conditioned, so one factorisation per
    iteration is dropped on the device; the result must still meet the oracle (which never drops any)."""
    import dataclasses
    cfg = dataclasses.replace(scaled(CONFIGS[3], m, n, rank=20, k=24, p=8),
                              spectrum=lambda i: 4.0 - i / 10.0)      # 4 .. 2.1 over a noise floor near 1
    A = workloads.build(cfg)
    A_dev = to_dev(A)
    _, _, _, info = ctx().rsvd_run(A_dev, cfg.k, cfg.p, q, seed=cfg.seed)
    assert info.skipped_reorth == expect
    run_and_compare(cfg, A_dev, A, q=q, note="adaptive schedule")


def test_ill_conditioned_panel_keeps_the_full_schedule():
    cfg = scaled(CONFIGS[2], 1500, 400, k=40, p=24)       # 0.9^i: condition ~ 850 over the 64 sketched directions
    A = workloads.build(cfg)
    _, _, _, info = ctx().rsvd_run(to_dev(A), cfg.k, cfg.p, 2, seed=cfg.seed)
    assert info.skipped_reorth == 0
    cfg1 = scaled(CONFIGS[1], 300, 200, rank=9, k=9, p=5)  # rank-deficient sketch: never dropped
    A1 = workloads.build(cfg1)
    _, _, _, info = ctx().rsvd_run(to_dev(A1), cfg1.k, cfg1.p, 2, seed=0)
    assert info.skipped_reorth == 0 and info.refilled_columns + info.raised_pivots > 0


@pytest.mark.parametrize("dt", ["f32", "f64"])
def test_degenerate_inputs(dt):
    """Zero and constant matrices, a single row, a single column, 1 x 1: finite outputs, the singular values of the
    textbook answer, orthonormal right vectors (the left vectors of singular values that are numerically zero
    come back as zero columns); nothing hangs and nothing is flagged."""
    say("degenerate", dt)
    T = np.float32 if dt == "f32" else np.float64
    eps = parity.EPS[dt]
    c = ctx()

    def run(A, k, p, q):
        S, U, Vt, info = c.rsvd_run(to_dev(np.ascontiguousarray(A.astype(T))), k, p, q, seed=1)
        S, U, Vt = (to_np(t).astype(np.float64) for t in (S, U, Vt))
        assert info.status == 0
        assert np.isfinite(S).all() and np.isfinite(U).all() and np.isfinite(Vt).all()
        return S, U, Vt, info

    S, U, Vt, info = run(np.zeros((300, 200)), 5, 5, 2)
    assert (S == 0).all() and info.refilled_columns > 0
    assert parity.orthonormality(Vt.T) <= 50 * eps                 # arbitrary, but orthonormal
    assert (U == 0).all()                                          # no direction belongs to a zero singular value
    S, U, Vt, _ = run(np.full((300, 200), 3.0), 4, 4, 1)
    assert S[0] == pytest.approx(3.0 * np.sqrt(300 * 200), rel=20 * eps) and (S[1:] <= 1e3 * eps * S[0]).all()
    assert np.abs(np.abs(U[:, 0]) - 1 / np.sqrt(300)).max() <= 50 * eps
    x = workloads.gaussian_matrix(500, 1, 5)
    S, U, Vt, _ = run(x, 1, 0, 2)                                  # one column
    assert S[0] == pytest.approx(np.linalg.norm(x.astype(T).astype(np.float64)), rel=20 * eps)
    assert abs(abs(Vt[0, 0]) - 1) <= 10 * eps
    S, U, Vt, _ = run(x.T, 1, 0, 2)                                # one row
    assert S[0] == pytest.approx(np.linalg.norm(x.astype(T).astype(np.float64)), rel=20 * eps)
    assert abs(abs(U[0, 0]) - 1) <= 10 * eps
    S, U, Vt, _ = run(np.array([[-2.5]]), 1, 0, 3)
    assert S[0] == pytest.approx(2.5, rel=10 * eps) and U[0, 0] * Vt[0, 0] == pytest.approx(-1.0, rel=10 * eps)


def test_two_contexts_on_two_streams():
    """Calls on different contexts, workspaces and streams may overlap in time: each gives, bit for bit, what it
    gives alone."""
    import torch
    from paper_2110_03423_amd import Rsvd, F32
    say("two streams")
    cfgs = [scaled(CONFIGS[2], 6000, 1500, k=48, p=16), scaled(CONFIGS[5], 3000, 1400, k=150, p=10)]
    As = [to_dev(workloads.build(cf)) for cf in cfgs]
    alone = []
    for A, cf in zip(As, cfgs):
        S, U, Vt, info = ctx().rsvd_run(A, cf.k, cf.p, 2, seed=7)
        assert info.status == 0
        alone.append([t.clone() for t in (S, U, Vt)])
    ctxs = [Rsvd(0), Rsvd(0)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    wss = [torch.empty(c.workspace_bytes(F32, cf.m, cf.n, cf.k, cf.p), dtype=torch.uint8, device="cuda:0")
           for c, cf in zip(ctxs, cfgs)]
    torch.cuda.synchronize()
    for rep in range(3):
        res = []
        for c, st, ws, A, cf in zip(ctxs, streams, wss, As, cfgs):
            with torch.cuda.stream(st):
                res.append(c.rsvd_run(A, cf.k, cf.p, 2, seed=7, workspace=ws, want_info=False))
        torch.cuda.synchronize()
        for got, want in zip(res, alone):
            assert all(torch.equal(g, w) for g, w in zip(got[:3], want)), f"repetition {rep}"
