"""Host-side logic of the C ABI without a GPU: a planning context (RSVD_DEVICE_NONE) sizes
workspaces and runs every argument check of the entry points, then declines to launch.
The fake device pointers below are never dereferenced: validation only compares them
with NULL and looks at their alignment."""
import ctypes as C

import pytest

from paper_2110_03423_amd import binding
from paper_2110_03423_amd.binding import F32, F64, JOB_S, JOB_SV, JOB_SUV, ERR_NO_DEVICE
import workloads

UNSUPPORTED = 4
PTR = C.c_void_p(1 << 20)          # "device memory", 256-byte aligned


@pytest.fixture(scope="module")
def plan():
    import os
    if not os.path.exists(binding.library_path()):
        from paper_2110_03423_amd import build
        build.build_library()
    return binding.Rsvd(device=None)


def _run(lib, h, **kw):
    a = dict(stream=None, dtype=F32, job=JOB_SUV, m=1000, n=400, A=PTR, lda=400, k=20, p=10, q=2, seed=0,
             S=PTR, U=PTR, ldu=20, Vt=PTR, ldvt=400, ws=PTR, ws_bytes=1 << 40, info=None)
    a.update(kw)
    return lib.rsvd_run(h, a["stream"], a["dtype"], a["job"], a["m"], a["n"], a["A"], a["lda"], a["k"], a["p"],
                        a["q"], a["seed"], a["S"], a["U"], a["ldu"], a["Vt"], a["ldvt"], a["ws"], a["ws_bytes"],
                        a["info"])


def test_planning_context_sizes_the_five_configurations(plan):
    for cfg in workloads.CONFIGS.values():
        dt = F32 if cfg.dtype == "f32" else F64
        es = 4 if cfg.dtype == "f32" else 8
        need = plan.workspace_bytes(dt, cfg.m, cfg.n, cfg.k, cfg.p, cfg.q)
        panels = 2 * (cfg.m + cfg.n) * cfg.l * es                      # the four ping-pong panels alone
        assert need % 256 == 0 and panels < need < 2 * panels + (64 << 20), (cfg.name, need, panels)
    # grows with the sketch width, does not depend on q or on the job
    sizes = [plan.workspace_bytes(F32, 5000, 3000, k, 8) for k in (8, 56, 120, 300, 600)]
    assert sizes == sorted(sizes) and len(set(sizes)) == len(sizes)
    assert plan.workspace_bytes(F32, 5000, 3000, 56, 8, q=0) == plan.workspace_bytes(F32, 5000, 3000, 56, 8, q=5)
    assert plan.workspace_bytes(F32, 5000, 3000, 56, 8, job=JOB_S) == plan.workspace_bytes(F32, 5000, 3000, 56, 8)
    # a batch is that many workspaces back to back
    one = plan.workspace_bytes(F64, 2000, 500, 16, 16)
    out = C.c_size_t()
    assert plan.lib.rsvd_workspace_bytes_batched(plan.h, F64, 7, 2000, 500, 16, 16, 1, JOB_SUV, C.byref(out)) == 0
    assert out.value == 7 * one


def test_workspace_query_argument_checks(plan):
    lib, h, out = plan.lib, plan.h, C.c_size_t()
    ok = dict(dtype=F32, m=100, n=50, k=5, p=5, q=1, job=JOB_SUV)

    def call(**kw):
        a = dict(ok, **kw)
        return lib.rsvd_workspace_bytes(h, a["dtype"], a["m"], a["n"], a["k"], a["p"], a["q"], a["job"], C.byref(out))
    assert call() == 0
    assert call(dtype=7) == -2 and call(m=0) == -3 and call(n=0) == -4 and call(k=0) == -5
    assert call(p=-1) == -6 and call(k=30, p=21) == -6 and call(k=25, p=25) == 0      # k + p <= min(m, n)
    assert call(q=-1) == -7 and call(job=3) == -8
    assert lib.rsvd_workspace_bytes(h, F32, 100, 50, 5, 5, 1, JOB_SUV, None) == -9
    assert lib.rsvd_workspace_bytes_batched(h, F32, 0, 100, 50, 5, 5, 1, JOB_SUV, C.byref(out)) == -3
    assert lib.rsvd_workspace_bytes_batched(h, F32, 2, 100, 0, 5, 5, 1, JOB_SUV, C.byref(out)) == -5


def test_rsvd_run_checks_every_argument_then_declines_to_launch(plan):
    lib, h = plan.lib, plan.h
    assert _run(lib, h) == ERR_NO_DEVICE                                # all arguments valid, nothing launched
    assert b"nothing was launched" in lib.rsvd_status_string(ERR_NO_DEVICE)
    assert _run(lib, None) == -1
    assert _run(lib, h, dtype=2) == -3 and _run(lib, h, job=-1) == -4
    assert _run(lib, h, m=0) == -5 and _run(lib, h, n=0) == -6
    assert _run(lib, h, A=None) == -7 and _run(lib, h, lda=399) == -8
    assert _run(lib, h, k=0) == -9
    assert _run(lib, h, p=-1) == -10 and _run(lib, h, k=300, p=101) == -10
    assert _run(lib, h, q=-1) == -11
    assert _run(lib, h, S=None) == -13
    assert _run(lib, h, U=None) == -14 and _run(lib, h, ldu=19) == -15
    assert _run(lib, h, Vt=None) == -16 and _run(lib, h, ldvt=399) == -17
    # outputs that the job does not ask for may be missing
    assert _run(lib, h, job=JOB_S, U=None, Vt=None, ldu=0, ldvt=0) == ERR_NO_DEVICE
    assert _run(lib, h, job=JOB_SV, U=None, ldu=0) == ERR_NO_DEVICE
    # workspace: present, 256-byte aligned, large enough
    need = plan.workspace_bytes(F32, 1000, 400, 20, 10)
    assert _run(lib, h, ws=None) == -18 and _run(lib, h, ws=C.c_void_p((1 << 20) + 64)) == -18
    assert _run(lib, h, ws_bytes=need - 1) == -19 and _run(lib, h, ws_bytes=need) == ERR_NO_DEVICE
    # sketch widths beyond what the small-SVD kernels cover
    assert _run(lib, h, dtype=F32, m=4000, n=4000, lda=4000, ldvt=4000, k=1500, p=100, ldu=1500) == UNSUPPORTED
    assert _run(lib, h, dtype=F64, m=4000, n=4000, lda=4000, ldvt=4000, k=800, p=0, ldu=800) == UNSUPPORTED
    assert _run(lib, h, dtype=F64, m=4000, n=4000, lda=4000, ldvt=4000, k=700, p=0, ldu=700) == ERR_NO_DEVICE


def test_static_scratch_entry_point_checks_size_and_arguments(plan):
    """rsvd_run_static on the planning context: the size check against the 32 MiB buffer and the argument checks
    of rsvd_run (positions 1-17 are the same), then the refusal to launch."""
    lib, h = plan.lib, plan.h
    SCRATCH_LIMIT = 6

    def call(**kw):
        a = dict(dtype=F32, job=JOB_SUV, m=1000, n=400, A=PTR, lda=400, k=20, p=10, q=2, S=PTR, U=PTR, ldu=20,
                 Vt=PTR, ldvt=400)
        a.update(kw)
        return lib.rsvd_run_static(h, None, a["dtype"], a["job"], a["m"], a["n"], a["A"], a["lda"], a["k"], a["p"],
                                   a["q"], 0, a["S"], a["U"], a["ldu"], a["Vt"], a["ldvt"], None)
    limit = lib.rsvd_static_scratch_bytes()
    assert limit == 32 << 20
    assert call() == ERR_NO_DEVICE
    assert call(A=None) == -7 and call(lda=399) == -8 and call(k=0) == -9 and call(S=None) == -13
    assert lib.rsvd_run_static(None, None, F32, JOB_SUV, 10, 10, PTR, 10, 2, 2, 1, 0, PTR, PTR, 2, PTR, 10, None) == -1
    # configuration 2 (the paper's benchmark shape) fits, configuration 3 does not
    c2, c3 = workloads.CONFIGS[2], workloads.CONFIGS[3]
    assert plan.workspace_bytes(F32, c2.m, c2.n, c2.k, c2.p) <= limit < plan.workspace_bytes(F32, c3.m, c3.n, c3.k, c3.p)
    assert call(m=c2.m, n=c2.n, lda=c2.n, ldvt=c2.n, k=c2.k, p=c2.p, ldu=c2.k) == ERR_NO_DEVICE
    assert call(m=c3.m, n=c3.n, lda=c3.n, ldvt=c3.n, k=c3.k, p=c3.p, ldu=c3.k) == SCRATCH_LIMIT
    assert b"static scratch" in lib.rsvd_status_string(SCRATCH_LIMIT)


def test_batched_entry_point_reports_positions_of_its_own_prototype(plan):
    lib, h = plan.lib, plan.h

    def call(**kw):
        a = dict(dtype=F32, job=JOB_SUV, batch=3, m=600, n=200, A=PTR, lda=200, stride_a=600 * 200, k=12, p=4, q=1,
                 S=PTR, stride_s=12, U=PTR, ldu=12, stride_u=600 * 12, Vt=PTR, ldvt=200, stride_vt=12 * 200,
                 ws=PTR, ws_bytes=1 << 40)
        a.update(kw)
        return lib.rsvd_run_batched(h, None, a["dtype"], a["job"], a["batch"], a["m"], a["n"], a["A"], a["lda"],
                                    a["stride_a"], a["k"], a["p"], a["q"], 0, a["S"], a["stride_s"], a["U"], a["ldu"],
                                    a["stride_u"], a["Vt"], a["ldvt"], a["stride_vt"], a["ws"], a["ws_bytes"], None)
    assert call() == ERR_NO_DEVICE
    assert call(batch=0) == -5 and call(m=0) == -6 and call(n=0) == -7 and call(A=None) == -8 and call(lda=10) == -9
    assert call(stride_a=600 * 200 - 1) == -10                          # problems would overlap
    assert call(k=0) == -11 and call(p=500) == -12 and call(q=-1) == -13
    assert call(S=None) == -15 and call(stride_s=11) == -16
    assert call(U=None) == -17 and call(ldu=11) == -18 and call(stride_u=10) == -19
    assert call(Vt=None) == -20 and call(ldvt=199) == -21 and call(stride_vt=10) == -22
    assert call(ws=None) == -23
    one = plan.workspace_bytes(F32, 600, 200, 12, 4)
    assert call(ws_bytes=3 * one - 1) == -24 and call(ws_bytes=3 * one) == ERR_NO_DEVICE
    # a batch needs the single-workgroup Cholesky and Jacobi kernels: l <= 128
    assert call(m=2000, n=2000, lda=2000, ldvt=2000, stride_a=4000000, stride_vt=2000 * 130, k=129, p=0, ldu=129,
                stride_s=129, stride_u=2000 * 129) == UNSUPPORTED
    assert call(dtype=F64, k=120, p=9, ldu=120, stride_s=120, stride_u=600 * 120, stride_vt=120 * 200) == UNSUPPORTED
    assert call(dtype=F64, k=120, p=8, ldu=120, stride_s=120, stride_u=600 * 120, stride_vt=120 * 200) == ERR_NO_DEVICE
    assert call(dtype=F64, k=90, p=7, ldu=90, stride_s=90, stride_u=600 * 90, stride_vt=90 * 200) == ERR_NO_DEVICE


def test_stage_entry_points_check_then_decline(plan):
    lib, h = plan.lib, plan.h
    big = 1 << 40
    assert lib.rsvd_stage_sketch(h, None, F32, 1, 0, 100, 20, PTR, 20) == ERR_NO_DEVICE
    assert lib.rsvd_stage_sketch(h, None, F32, 1, 0, 100, 20, PTR, 19) == -9
    assert lib.rsvd_stage_sketch(h, None, F32, 1, 0, 0, 20, None, 0) == 0            # empty: nothing to do
    assert lib.rsvd_stage_gemm_an(h, None, F64, 300, 100, 10, PTR, 100, PTR, 10, PTR, 10, PTR, big) == ERR_NO_DEVICE
    assert lib.rsvd_stage_gemm_an(h, None, F64, 300, 100, 101, PTR, 100, PTR, 101, PTR, 101, PTR, big) == -6
    assert lib.rsvd_stage_gemm_atn(h, None, F64, 300, 100, 10, PTR, 100, PTR, 9, PTR, 10, PTR, big) == -10
    assert lib.rsvd_stage_orth(h, None, F32, 500, 40, PTR, 40, None, 0, 16, PTR, big, None) == ERR_NO_DEVICE
    assert lib.rsvd_stage_orth(h, None, F32, 30, 40, PTR, 40, None, 0, 16, PTR, big, None) == -5
    assert lib.rsvd_stage_small_svd(h, None, F32, 500, 40, PTR, 40, PTR, PTR, PTR, 40, 0, PTR, big, None) == ERR_NO_DEVICE
    assert lib.rsvd_stage_small_svd(h, None, F32, 500, 40, PTR, 40, PTR, PTR, PTR, 39, 0, PTR, big, None) == -11
    assert lib.rsvd_stage_jacobi(h, None, F64, 64, PTR, PTR, PTR, PTR, PTR, big, None) == ERR_NO_DEVICE
    assert lib.rsvd_stage_jacobi(h, None, F64, 64, PTR, None, PTR, PTR, PTR, big, None) == -6
    assert lib.rsvd_stage_lift(h, None, F32, 500, 40, 30, PTR, 40, PTR, 30, PTR, 30, 0, None, 0) == ERR_NO_DEVICE
    assert lib.rsvd_stage_lift(h, None, F32, 500, 40, 41, PTR, 40, PTR, 41, PTR, 41, 0, None, 0) == -6
    assert lib.rsvd_stage_lift(h, None, F32, 500, 40, 30, PTR, 40, PTR, 30, PTR, 499, 1, None, 0) == -12   # transposed: ldu >= m


def test_stage_workspace_is_sized_by_the_panel_alone(plan):
    lib, h, out = plan.lib, plan.h, C.c_size_t()
    assert lib.rsvd_stage_workspace_bytes(h, F32, 100000, 120, C.byref(out)) == 0
    panels = 2 * 100000 * 120 * 4
    assert out.value % 256 == 0 and panels < out.value < panels + (64 << 20)      # no term grows with rows^2
    assert out.value <= plan.workspace_bytes(F32, 100000, 100000, 120, 0)           # the full-problem figure also covers it
    need = out.value
    assert lib.rsvd_stage_orth(h, None, F32, 100000, 120, PTR, 120, None, 0, 16, PTR, need, None) == ERR_NO_DEVICE
    assert lib.rsvd_stage_orth(h, None, F32, 100000, 120, PTR, 120, None, 0, 16, PTR, need - 1, None) == -12
    assert lib.rsvd_stage_small_svd(h, None, F32, 100000, 120, PTR, 120, PTR, PTR, PTR, 120, 0, PTR, need, None) == ERR_NO_DEVICE
    assert lib.rsvd_stage_workspace_bytes(h, F64, 64, 64, C.byref(out)) == 0
    assert lib.rsvd_stage_jacobi(h, None, F64, 64, PTR, PTR, PTR, PTR, PTR, out.value, None) == ERR_NO_DEVICE
    assert lib.rsvd_stage_workspace_bytes(h, 3, 64, 64, C.byref(out)) == -2
    assert lib.rsvd_stage_workspace_bytes(h, F64, 0, 64, C.byref(out)) == -3
    assert lib.rsvd_stage_workspace_bytes(h, F64, 64, 65, C.byref(out)) == -4
    assert lib.rsvd_stage_workspace_bytes(h, F64, 64, 64, None) == -5


def test_no_such_device_is_an_error(plan):
    h = C.c_void_p()
    lib = plan.lib
    assert lib.rsvd_create(C.byref(h), -7) == -2 and not h.value
    assert lib.rsvd_create(None, 0) == -1
