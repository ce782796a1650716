"""rsvd_run under HIP graph capture: with a caller-owned workspace and no diagnostics
the call allocates nothing, never synchronises and clears its scratch with kernels,
so a serving loop can record it once and replay it.  Every replay is checked against
the eager result (the path is deterministic, so the comparison is bit for bit), with
eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import workloads
from workloads import CONFIGS, scaled
from gpu_util import ctx, to_dev, say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cid,m,n,k,p,q", [
    (1, 512, 256, 10, 10, 2),        # rank deficient: replacement columns inside the graph
    (2, 3000, 700, 48, 16, 2),       # LDS-resident Cholesky and Jacobi
    (5, 2500, 1200, 150, 10, 1),     # blocked Cholesky and block Jacobi (several hundred launches)
])
def test_graph_replay_matches_eager(cid, m, n, k, p, q):
    say("graph", cid, m, n, k, p, q)
    cfg = scaled(CONFIGS[cid], m, n, k=k, p=p)
    A = to_dev(workloads.build(cfg))
    c = ctx()
    dt = 0 if cfg.dtype == "f32" else 1
    ws = c.workspace(dt, m, n, k, p)
    out = (torch.empty(k, dtype=A.dtype, device=A.device), torch.empty((m, k), dtype=A.dtype, device=A.device),
           torch.empty((k, n), dtype=A.dtype, device=A.device))
    # eager reference (also the first call of every kernel, outside the capture)
    _, _, _, info = c.rsvd_run(A, k, p, q, seed=cfg.seed, workspace=ws, out=out)
    assert info.status == 0
    torch.cuda.synchronize()
    ref = [t.clone() for t in out]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        c.rsvd_run(A, k, p, q, seed=cfg.seed, workspace=ws, want_info=False, out=out)
    torch.cuda.synchronize()

    for rep in range(4):
        # eager work between the replays: wipe the outputs and dirty the workspace
        for t in out:
            t.fill_(float("nan"))
        ws.fill_(0x5A if rep % 2 else 0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, want in zip(("S", "U", "Vt"), out, ref):
            assert torch.equal(got, want), f"replay {rep}: {name} differs from the eager call"
