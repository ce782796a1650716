"""rsvd_run_static: the entry point for callers that cannot allocate (it works in a static
buffer inside the library).  It runs the same kernels over the same workspace layout as
rsvd_run, and the path is deterministic, so its results must equal those of rsvd_run bit
for bit -- on two calls in a row through the C ABI, the second on a smaller input, so that
whatever the first call left in the shared buffer is seen not to matter."""
import ctypes as C

import numpy as np
import pytest
import torch

import workloads
from workloads import CONFIGS, scaled
from paper_2110_03423_amd import binding
from gpu_util import ctx, to_dev, say

pytestmark = pytest.mark.gpu

SCRATCH_LIMIT = 6


def _call_static(c, A, k, p, q, seed, out, info):
    """Straight through ctypes: nothing but pointers and sizes crosses the boundary."""
    S, U, Vt = out
    m, n = A.shape
    dt = 0 if A.dtype == torch.float32 else 1
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    return c.lib.rsvd_run_static(c.h, stream, dt, binding.JOB_SUV, m, n, C.c_void_p(A.data_ptr()), A.stride(0),
                                 k, p, q, seed, C.c_void_p(S.data_ptr()), C.c_void_p(U.data_ptr()), U.stride(0),
                                 C.c_void_p(Vt.data_ptr()), Vt.stride(0), C.byref(info) if info is not None else None)


def test_static_scratch_entry_matches_rsvd_run_twice_in_a_row():
    c = ctx()
    assert c.lib.rsvd_static_scratch_bytes() == 32 << 20
    cases = [scaled(CONFIGS[2], 5000, 1500, k=64, p=16),      # ~20 MiB of workspace: most of the buffer
             scaled(CONFIGS[1], 300, 200, rank=9, k=9, p=7)]  # smaller, other dtype, replacement columns
    for cfg in cases:
        say("static", cfg.name, cfg.dtype, cfg.k, cfg.p, cfg.q)
        A = to_dev(workloads.build(cfg))
        m, n, k = cfg.m, cfg.n, cfg.k
        dt = 0 if cfg.dtype == "f32" else 1
        assert c.workspace_bytes(dt, m, n, cfg.k, cfg.p) <= 32 << 20
        want = c.rsvd_run(A, cfg.k, cfg.p, cfg.q, seed=cfg.seed)
        torch.cuda.synchronize()
        out = (torch.full((k,), float("nan"), dtype=A.dtype, device=A.device),
               torch.full((m, k), float("nan"), dtype=A.dtype, device=A.device),
               torch.full((k, n), float("nan"), dtype=A.dtype, device=A.device))
        info = binding._Info()
        rc = _call_static(c, A, cfg.k, cfg.p, cfg.q, cfg.seed, out, info)
        assert rc == 0 and info.status == 0
        assert info.jacobi_sweeps == want[3].jacobi_sweeps and info.refilled_columns == want[3].refilled_columns
        for name, got, ref in zip(("S", "U", "Vt"), out, want[:3]):
            assert torch.equal(got, ref), f"{cfg.name}: {name} differs from rsvd_run"
        # and without diagnostics (fully asynchronous)
        for t in out:
            t.fill_(float("nan"))
        assert _call_static(c, A, cfg.k, cfg.p, cfg.q, cfg.seed, out, None) == 0
        torch.cuda.synchronize()
        for name, got, ref in zip(("S", "U", "Vt"), out, want[:3]):
            assert torch.equal(got, ref), f"{cfg.name}: {name} differs from rsvd_run (info = NULL)"


def test_static_scratch_entry_rejects_what_does_not_fit():
    c = ctx()
    cfg = CONFIGS[3]                                        # 122 MiB of workspace
    A = torch.zeros((8, 8), dtype=torch.float32, device="cuda:0")     # never read: the size check comes first
    out = (A, A, A)
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = c.lib.rsvd_run_static(c.h, stream, 0, binding.JOB_SUV, cfg.m, cfg.n, C.c_void_p(A.data_ptr()), cfg.n,
                               cfg.k, cfg.p, cfg.q, 0, C.c_void_p(A.data_ptr()), C.c_void_p(A.data_ptr()), cfg.k,
                               C.c_void_p(A.data_ptr()), cfg.n, None)
    assert rc == SCRATCH_LIMIT
    assert b"static scratch" in c.lib.rsvd_status_string(rc)
