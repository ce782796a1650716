"""GPU parity of rsvd_run_batched: many equal-shaped problems per launch (the use
the paper's clustering application makes of the solver), every problem against the
CPU oracle with its own seed, and against rsvd_run on the same matrix."""
import dataclasses

import numpy as np
import pytest

import workloads
from workloads import CONFIGS, scaled
from oracle import rsvd as orc
import parity
from gpu_util import ctx, to_np, say

pytestmark = pytest.mark.gpu


def _problems(base, batch):
    """`batch` matrices of one shape built by the recipe of `base` with different factor seeds."""
    out = []
    for b in range(batch):
        cfg = dataclasses.replace(base, cid=base.cid + 10 * b)       # seeds 1000 + cid, 2000 + cid, 3000 + cid
        out.append(workloads.build(cfg))
    return np.stack(out)


def _check_problem(b, cfg, A_host, S, U, Vt, seed, q):
    dt, m, n, k, p = cfg.dtype, cfg.m, cfg.n, cfg.k, cfg.p
    o = orc.rsvd(A_host, k, p, q, seed, cfg.np_dtype)
    # (a cluster of singular values that may straddle k is compared on the values only here)
    res = parity.check_triplets(S, U, Vt, o.S, o.U, o.Vt, dt, m, n)
    eps = parity.EPS[dt]
    ns = int(parity.significant(o.S, dt, m, n).sum())
    err_g = orc.reconstruction_error(A_host, U, S, Vt)
    err_o = orc.reconstruction_error(A_host, o.U, o.S, o.Vt)
    normA = float(np.sqrt(np.sum(A_host.astype(np.float64) ** 2)))
    assert err_g <= 1.01 * err_o + 50 * eps * normA, (b, err_g, err_o)
    assert parity.orthonormality(U[:, :ns]) <= parity.jacobi_tol(cfg.l, dt)
    assert parity.orthonormality(Vt[:ns].T) <= parity.jacobi_tol(cfg.l, dt)
    return res["sv_rel_max"]


CASES = [
    # base config (shape, spectrum), batch, q
    (scaled(CONFIGS[2], 700, 300, k=20, p=12), 5, 2),            # fp32, l = 32, split-K products
    (scaled(CONFIGS[1], 200, 160, rank=12, k=10, p=6), 7, 1),    # fp64, exact recovery, rank-deficient sketch
    (scaled(CONFIGS[3], 2000, 250, rank=25, k=40, p=8), 3, 2),   # fp32, l = 48, noisy tail
    (scaled(CONFIGS[4], 500, 400, rank=64, k=64, p=32), 4, 1),   # fp64, l = 96: largest fp64 order held in LDS whole
    (scaled(CONFIGS[4], 600, 450, rank=80, k=80, p=25), 3, 1),   # fp64, l = 105: rotations accumulated in global memory
    (scaled(CONFIGS[4], 700, 500, rank=100, k=100, p=28), 3, 2), # fp64, l = 128: largest order of the batched path
    (scaled(CONFIGS[2], 333, 129, k=7, p=6), 9, 0),              # odd everything: scalar load paths, q = 0
    (scaled(CONFIGS[5], 600, 300, rank=64, k=100, p=28), 3, 1),  # fp32, l = 128: largest order of the batched path
]


@pytest.mark.parametrize("base,batch,q", CASES, ids=lambda v: getattr(v, "name", str(v)))
def test_batched_matches_oracle_and_single_calls(base, batch, q):
    import torch
    say("batched", base.name, "batch", batch, "q", q)
    A = _problems(base, batch)
    A_dev = torch.from_numpy(A).to("cuda:0")
    c = ctx()
    seed = 40
    S, U, Vt, info = c.rsvd_run_batched(A_dev, base.k, base.p, q, seed=seed)
    torch.cuda.synchronize()
    assert info.status == 0
    S, U, Vt = (to_np(t).astype(np.float64) for t in (S, U, Vt))
    worst = 0.0
    for b in range(batch):
        worst = max(worst, _check_problem(b, base, A[b], S[b], U[b], Vt[b], seed + b, q))
        # the same matrix through rsvd_run with the same seed: same Omega, same algorithm; only the
        # split of the long sums may differ, so the singular values agree to rounding
        S1, U1, Vt1, _ = c.rsvd_run(A_dev[b], base.k, base.p, q, seed=seed + b)
        S1 = to_np(S1).astype(np.float64)
        sig = parity.significant(S1, base.dtype, base.m, base.n)
        tol = 200 * parity.EPS[base.dtype] * np.sqrt(max(base.m, base.n))
        assert (np.abs(S[b] - S1)[sig] <= tol * S1[0]).all(), b
    say("  worst relative singular value error", worst, "sweeps", info.jacobi_sweeps)


def test_batch_mixes_schedules():
    """The adaptive re-orthonormalisation is decided per problem on the device: a batch that holds a
    well-conditioned matrix (drops a factorisation) next to an ill-conditioned one (keeps all) must get both right."""
    import torch
    flat = dataclasses.replace(scaled(CONFIGS[3], 1500, 300, rank=20, k=24, p=8), spectrum=lambda i: 4.0 - i / 10.0)
    steep = dataclasses.replace(scaled(CONFIGS[2], 1500, 300, k=24, p=8), dtype="f32")
    A = np.stack([workloads.build(flat), workloads.build(steep), workloads.build(dataclasses.replace(flat, cid=33))])
    A_dev = torch.from_numpy(A).to("cuda:0")
    c = ctx()
    S, U, Vt, info = c.rsvd_run_batched(A_dev, 24, 8, 2, seed=5)
    torch.cuda.synchronize()
    assert info.status == 0 and info.skipped_reorth == 1
    S, U, Vt = (to_np(t).astype(np.float64) for t in (S, U, Vt))
    for b, cfg in enumerate((flat, steep, flat)):
        _check_problem(b, cfg, A[b], S[b], U[b], Vt[b], 5 + b, 2)
    # each problem on its own takes the schedule its own conditioning calls for
    assert c.rsvd_run(A_dev[0], 24, 8, 2, seed=5)[3].skipped_reorth == 1
    assert c.rsvd_run(A_dev[1], 24, 8, 2, seed=6)[3].skipped_reorth == 0


def test_batched_strides_jobs_and_batch_of_one():
    import torch
    from paper_2110_03423_amd import JOB_S, JOB_SV
    base = scaled(CONFIGS[2], 300, 200, k=8, p=8)
    A = _problems(base, 4)
    c = ctx()
    # problems padded apart: strides larger than the matrices
    big = torch.zeros((4, 310, 208), dtype=torch.float32, device="cuda:0")
    big[:, :300, :200] = torch.from_numpy(A).to("cuda:0")
    S0, U0, Vt0, _ = c.rsvd_run_batched(torch.from_numpy(A).to("cuda:0"), 8, 8, 2, seed=3)
    S1, U1, Vt1, _ = c.rsvd_run_batched(big[:, :300, :200], 8, 8, 2, seed=3)
    assert torch.equal(S0, S1) and torch.equal(U0, U1) and torch.equal(Vt0, Vt1)
    S2, U2, Vt2, _ = c.rsvd_run_batched(torch.from_numpy(A).to("cuda:0"), 8, 8, 2, seed=3, job=JOB_S)
    assert U2 is None and Vt2 is None and torch.equal(S0, S2)
    S3, U3, Vt3, _ = c.rsvd_run_batched(torch.from_numpy(A).to("cuda:0"), 8, 8, 2, seed=3, job=JOB_SV)
    assert U3 is None and torch.equal(Vt0, Vt3)
    # a batch of one is rsvd_run
    Sb, Ub, Vtb, _ = c.rsvd_run_batched(torch.from_numpy(A[:1]).to("cuda:0"), 8, 8, 2, seed=3)
    Ss, Us, Vts, _ = c.rsvd_run(torch.from_numpy(A[0]).to("cuda:0"), 8, 8, 2, seed=3)
    assert torch.equal(Sb[0], Ss) and torch.equal(Ub[0], Us) and torch.equal(Vtb[0], Vts)


def test_batched_rejects_what_it_cannot_do():
    import torch
    from paper_2110_03423_amd.binding import RsvdError
    c = ctx()
    A = torch.zeros((2, 400, 300), dtype=torch.float32, device="cuda:0")
    with pytest.raises(RsvdError) as e:
        c.rsvd_run_batched(A, 120, 40, 1)                     # l = 160: beyond the single-workgroup kernels
    assert e.value.code == 4
    with pytest.raises(RsvdError) as e:
        c.rsvd_run_batched(A.double(), 100, 29, 1)            # l = 129 in fp64 likewise
    assert e.value.code == 4
    with pytest.raises(RsvdError) as e:
        c.rsvd_run_batched(A, 200, 200, 1)                    # k + p > min(m, n): caught when the workspace is sized
    assert e.value.code == -7
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(RsvdError) as e:
        c.rsvd_run_batched(A, 200, 200, 1, workspace=ws)      # the same through rsvd_run_batched itself
    assert e.value.code == -12
    with pytest.raises(RsvdError) as e:
        c.rsvd_run_batched(A, 8, 8, 1, workspace=ws[:4096])   # workspace too small
    assert e.value.code == -24


def test_a_non_finite_problem_does_not_touch_its_neighbours():
    """One matrix of the batch holds a NaN: the call reports it, the other problems come out as they do alone."""
    import torch
    say("batched: one poisoned problem")
    c = ctx()
    A = np.stack([workloads.gaussian_matrix(400, 150, 60 + b, np.float32) for b in range(3)])
    clean = c.rsvd_run_batched(torch.from_numpy(A).to("cuda:0"), 10, 20, 2, seed=5)
    assert clean[3].status == 0
    A[1, 3, 3] = np.nan
    Ad = torch.from_numpy(A).to("cuda:0")
    from paper_2110_03423_amd import RsvdError
    with pytest.raises(RsvdError) as err:
        c.rsvd_run_batched(Ad, 10, 20, 2, seed=5)
    assert err.value.code == 1
    S, U, Vt, _ = c.rsvd_run_batched(Ad, 10, 20, 2, seed=5, want_info=False)
    torch.cuda.synchronize()
    for b in (0, 2):
        assert torch.equal(S[b], clean[0][b]) and torch.equal(U[b], clean[1][b]) and torch.equal(Vt[b], clean[2][b])
