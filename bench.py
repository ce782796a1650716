#!/usr/bin/env python3
"""Benchmark of the randomized SVD hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C]

A step is one full rsvd_run (sketch, range product, power iterations with
re-orthonormalisation, projection, small SVD, lift) on a synthetic matrix that
is already resident in HBM.  Prints one JSON line: wall time per call, the
roofline position of the kernel class that takes the most time (measured with
HIP events around every kernel launch in a second pass over the same steps),
and the CPU oracle timed on the host cores for the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_HBM = 8.0e12                                # B/s
PEAK_MFMA = {"f32": 157.3e12, "f64": 78.6e12}    # dense matrix FLOP/s
PEAK_VALU = {"f32": 157.3e12, "f64": 78.6e12}    # vector FLOP/s (256 CUs, 2.4 GHz)


# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script at configuration 2,
# scaled by the same counters on a plain 1 GiB copy (figures and commands: profiles/rsvd_run_cfg2_hbm_counters.md).
MEASURED_TRAFFIC = {2: {"cholesky": 0.14e6, "jacobi": 0.12e6, "gemm_atx": 103.8e6, "gemm_ax": 108.5e6,
                        "gram": 6.6e6, "apply_rinv": 7.1e6}}


def kernel_models(cfg):
    """Algorithmic flops and HBM bytes of ONE launch of each kernel class (unit: one launch)."""
    m, n, l, k = cfg.m, cfg.n, cfg.l, cfg.k
    sz = 4 if cfg.dtype == "f32" else 8
    models = {
        # products with A: read A once, read the skinny operand, write the result
        "gemm_ax": dict(flops=2.0 * m * n * l, bytes=(m * n + n * l + m * l) * sz, mfma=cfg.dtype),
        "gemm_atx": dict(flops=2.0 * m * n * l, bytes=(m * n + m * l + n * l) * sz, mfma=cfg.dtype),
        # small dense stages (latency / ALU bound): flops of the textbook algorithm
        "cholesky": dict(flops=(5.0 / 3.0) * l ** 3, bytes=2 * l * l * 8, alu="f64"),
        "sketch": dict(flops=None, bytes=n * l * sz),
    }
    return models


def per_launch_model(name, cfg, launches_per_call):
    """Flops / bytes of one launch for classes whose size alternates between m and n rows."""
    m, n, l, k = cfg.m, cfg.n, cfg.l, cfg.k
    sz = 4 if cfg.dtype == "f32" else 8
    q = cfg.q
    n_m, n_n = 2 * (q + 1), 2 * (q + 1)            # CholeskyQR rounds on m x l and on n x l panels
    if name == "gram":
        rows = (n_m * m + n_n * n) / (n_m + n_n)
        return dict(flops=2.0 * rows * l * l, bytes=rows * l * sz + l * l * 8, mfma="f64")
    if name == "apply_rinv":
        rows = (n_m * m + n_n * n) / (n_m + n_n)
        return dict(flops=2.0 * rows * l * l, bytes=2 * rows * l * sz + l * l * sz, mfma=cfg.dtype)
    if name == "lift":
        rows = (m + n) / 2.0
        return dict(flops=2.0 * rows * l * k, bytes=rows * (l + k) * sz, mfma=cfg.dtype)
    if name == "jacobi":
        # one sweep = l(l-1)/2 pair visits, each 3 inner products and 2 rotated column pairs of length l
        sweeps = launches_per_call if launches_per_call else 1
        return dict(flops=9.0 * l ** 3 * sweeps, bytes=3 * l * l * sz, alu=cfg.dtype)
    return kernel_models(cfg).get(name)


def roofline_for(name, avg_ms, cfg, sweeps=None):
    mod = per_launch_model(name, cfg, sweeps)
    if mod is None or avg_ms <= 0:
        return None
    t = avg_ms * 1e-3
    t_mem = mod["bytes"] / PEAK_HBM
    flops = mod.get("flops")
    if "mfma" in mod and flops and flops / PEAK_MFMA[mod["mfma"]] > t_mem:
        peak = PEAK_MFMA[mod["mfma"]]
        return dict(bound="mfma", achieved=flops / t / 1e12, peak=peak / 1e12, unit="TFLOP/s",
                    frac=flops / t / peak, traffic=None, kernel=name, avg_us=avg_ms * 1e3)
    if "alu" in mod and flops:
        # single-workgroup kernels on the serial path: priced against the vector peak
        # (one workgroup can use one of the 256 CUs: frac_one_cu prices it against that share)
        peak = PEAK_VALU[mod["alu"]]
        return dict(bound="alu", achieved=flops / t / 1e12, peak=peak / 1e12, unit="TFLOP/s",
                    frac=flops / t / peak, frac_one_cu=flops / t / (peak / 256.0), traffic=None, kernel=name,
                    avg_us=avg_ms * 1e3)
    return dict(bound="hbm", achieved=mod["bytes"] / t / 1e9, peak=PEAK_HBM / 1e9, unit="GB/s",
                frac=mod["bytes"] / t / PEAK_HBM, traffic=None, kernel=name, avg_us=avg_ms * 1e3)


def cpu_baseline(cfg, A_host, budget_s=20.0):
    """The oracle as it stands, on the host cores, on the same workload."""
    import numpy as np
    from oracle import rsvd as orc
    cores = len(os.sched_getaffinity(0))
    try:
        from threadpoolctl import threadpool_info
        nt = [d.get("num_threads") for d in threadpool_info() if d.get("user_api") == "blas"]
        if nt:
            cores = min(cores, max(nt))
    except Exception:
        pass
    runs, t_total = 0, 0.0
    while runs < 3 and t_total < budget_s:
        t0 = time.perf_counter()
        orc.rsvd(A_host, cfg.k, cfg.p, cfg.q, cfg.seed, cfg.np_dtype)
        t_total += time.perf_counter() - t0
        runs += 1
    return dict(value=t_total / runs * 1e3, unit="ms", cores=cores, kind="oracle",
                sample=f"{runs} full call(s) of the numpy fp64 oracle on the whole {cfg.m}x{cfg.n} workload")


def sweep(args):
    """Small-l runs at the shapes of configurations 3 and 5: one JSON line per (shape, k, p, q) with the
    achieved HBM rate of the two kernels that stream A (algorithmic bytes / HIP-event time per launch)."""
    import dataclasses
    import torch
    import workloads
    from paper_2110_03423_amd import Rsvd, F32, F64

    ctx = Rsvd(0)
    dev = "cuda:0"
    for cid in (3, 5):
        base = workloads.CONFIGS[cid]
        A = workloads.build(base, device=dev)
        dt = F32 if base.dtype == "f32" else F64
        for (k, p, q) in ((8, 8, 1), (24, 8, 1)):
            cfg = dataclasses.replace(base, k=k, p=p, q=q)
            ws = ctx.workspace(dt, cfg.m, cfg.n, k, p)
            out = (torch.empty(k, dtype=A.dtype, device=dev), torch.empty((cfg.m, k), dtype=A.dtype, device=dev),
                   torch.empty((k, cfg.n), dtype=A.dtype, device=dev))

            def step():
                ctx.rsvd_run(A, k, p, q, seed=cfg.seed, workspace=ws, want_info=False, out=out)

            for _ in range(args.warmup):
                step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                step()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / args.steps
            ctx.rsvd_profile_enable(True)
            for _ in range(args.steps):
                step()
            torch.cuda.synchronize()
            prof = ctx.rsvd_profile_read()
            ctx.rsvd_profile_enable(False)
            line = {"sweep": cfg.name, "dtype": cfg.dtype, "m": cfg.m, "n": cfg.n, "k": k, "p": p, "q": q,
                    "ms_per_call": round(ms, 4)}
            for name in ("gemm_ax", "gemm_atx"):
                tot, cnt = prof[name]
                r = roofline_for(name, tot / cnt, cfg)
                line[name] = dict(avg_us=round(tot / cnt * 1e3, 2), bound=r["bound"], achieved=round(r["achieved"], 1),
                                  unit=r["unit"], frac=round(r["frac"], 4))
            print(json.dumps(line), flush=True)
        del A
        torch.cuda.empty_cache()


def batched(args):
    """Batches of equal-shaped small problems (the clustering use of the solver): one JSON line per
    (shape, batch) with the time per problem of rsvd_run_batched and of a loop of rsvd_run calls."""
    import torch
    from paper_2110_03423_amd import Rsvd

    ctx = Rsvd(0)
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    cases = [  # m, n, k, p, q, dtype, batches
        (2000, 500, 16, 16, 1, torch.float32, (1, 16, 256)),
        (10000, 2000, 64, 16, 2, torch.float32, (1, 4, 16)),
        (4000, 1000, 32, 16, 2, torch.float64, (1, 16, 64)),
    ]
    for (m, n, k, p, q, tdt, batches) in cases:
        for batch in batches:
            # low-rank-plus-noise problems, a different one per slot
            r = 2 * (k + p)
            A = torch.randn((batch, m, r), dtype=tdt, device=dev, generator=gen) @ \
                (torch.randn((batch, r, n), dtype=tdt, device=dev, generator=gen) *
                 (0.9 ** torch.arange(r, dtype=tdt, device=dev))[None, :, None])
            A += 1e-3 * torch.randn(A.shape, dtype=tdt, device=dev, generator=gen)
            out_b = None

            def run_batched():
                nonlocal out_b
                out_b = ctx.rsvd_run_batched(A, k, p, q, seed=1, want_info=False)

            def run_loop():
                for b in range(batch):
                    ctx.rsvd_run(A[b], k, p, q, seed=1 + b, want_info=False)

            res = {}
            for name, fn in (("batched", run_batched), ("loop", run_loop)):
                for _ in range(args.warmup):
                    fn()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.steps):
                    fn()
                torch.cuda.synchronize()
                res[name] = (time.perf_counter() - t0) * 1e3 / args.steps
            print(json.dumps({"batched": f"{m}x{n}", "dtype": "f32" if tdt == torch.float32 else "f64", "k": k, "p": p,
                              "q": q, "batch": batch, "ms_per_problem_batched": round(res["batched"] / batch, 4),
                              "ms_per_problem_loop": round(res["loop"] / batch, 4),
                              "speedup": round(res["loop"] / res["batched"], 2)}), flush=True)
            del A
            torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration 1..5 (default 2)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--centered", action="store_true",
                    help="time rsvd_run_centered (PCA front end: implicit column centring) instead of rsvd_run")
    ap.add_argument("--sweep", action="store_true",
                    help="supplementary sweep instead of the benchmark: the shapes of configurations 3 and 5 with "
                         "(k, p, q) = (8, 8, 1) and (24, 8, 1), where the products with A are HBM bound")
    ap.add_argument("--batched", action="store_true",
                    help="supplementary: rsvd_run_batched on batches of small problems against a loop of rsvd_run calls")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (reference dispatch for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads
    from paper_2110_03423_amd import Rsvd, F32, F64

    if args.sweep:
        sweep(args)
        return
    if args.batched:
        batched(args)
        return
    cfg = workloads.CONFIGS[args.config]
    dev = "cuda:0"
    A = workloads.build(cfg, device=dev)
    ctx = Rsvd(0)
    dt = F32 if cfg.dtype == "f32" else F64
    ws = ctx.workspace(dt, cfg.m, cfg.n, cfg.k, cfg.p)
    out = (torch.empty(cfg.k, dtype=A.dtype, device=dev), torch.empty((cfg.m, cfg.k), dtype=A.dtype, device=dev),
           torch.empty((cfg.k, cfg.n), dtype=A.dtype, device=dev))

    mean_buf = torch.empty(cfg.n, dtype=A.dtype, device=dev)

    def step():
        ctx.rsvd_run(A, cfg.k, cfg.p, cfg.q, seed=cfg.seed, workspace=ws, want_info=False, out=out,
                     _mean=mean_buf if args.centered else None)

    for _ in range(args.warmup):
        step()
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    _, _, _, info = ctx.rsvd_run(A, cfg.k, cfg.p, cfg.q, seed=cfg.seed, workspace=ws, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # per-call spread (paper's protocol: mean and standard deviation over repeated runs)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
    for a, b in evs:
        a.record(); step(); b.record()
    torch.cuda.synchronize()
    per_call = np.array([a.elapsed_time(b) for a, b in evs])

    # supplementary: the same call recorded once as a HIP graph and replayed (what a serving loop would do;
    # the call allocates nothing and never synchronises when it gets its workspace and no diagnostics)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    del graph

    # second pass over the same steps with HIP events around every kernel launch
    ctx.rsvd_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = ctx.rsvd_profile_read()
    ctx.rsvd_profile_enable(False)
    kernels = {name: dict(ms_per_call=tot / args.steps, launches_per_call=cnt / args.steps,
                          avg_us=tot / cnt * 1e3) for name, (tot, cnt) in prof.items()}
    dominant = max(kernels, key=lambda kname: kernels[kname]["ms_per_call"])
    roof = roofline_for(dominant, kernels[dominant]["avg_us"] * 1e-3, cfg, info.jacobi_sweeps)
    if roof is not None:
        roof["traffic"] = MEASURED_TRAFFIC.get(args.config, {}).get(dominant)
    stage_roof = {}
    for name in kernels:
        r = roofline_for(name, kernels[name]["avg_us"] * 1e-3, cfg, info.jacobi_sweeps)
        if r is not None:
            stage_roof[name] = dict(bound=r["bound"], achieved=round(r["achieved"], 3), unit=r["unit"],
                                    frac=round(r["frac"], 4))

    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(cfg, A.cpu().numpy())

    line = {
        "metric": "rsvd_wall_time_ms",
        "value": round(ms_per_step, 4),
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_mean_std_10": [round(float(per_call.mean()), 4), round(float(per_call.std()), 4)],
        "ms_per_step_graph_replay": round(graph_ms, 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": cfg.name, "m": cfg.m, "n": cfg.n, "k": cfg.k, "p": cfg.p, "q": cfg.q,
                   "job": "S,U,Vt" + (" of the column-centred matrix" if args.centered else ""),
                   "jacobi_sweeps": info.jacobi_sweeps},
        "roofline": roof,
        "kernels": {kname: {a: round(b, 4) for a, b in v.items()} for kname, v in kernels.items()},
        "stage_roofline": stage_roof,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
