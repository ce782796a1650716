#!/usr/bin/env python3
"""Benchmark of the randomized SVD hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C]

A step is one full rsvd_run (sketch, range product, power iterations with
re-orthonormalisation, projection, small SVD, lift) on a synthetic matrix that
is already resident in HBM.  The default workload is configuration 5 (fp32
65536 x 16384, k = 512, p = 64, q = 1: the largest one and the one the matrix-core
target is stated on).  Prints one JSON line: wall time per call, the roofline
position of the kernel that takes the most time (measured with HIP events
around every kernel launch in a second pass over the same steps; the two
products with A are one kernel template and are priced together), the CPU
oracle timed on the host cores for the same workload, and under
`other_configs` the wall time and dominant kernel of the other four
configurations from shorter runs.
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

# Kernel classes that are one kernel template doing one job are priced together: the two products with A
# (Y = A X and Z = A^T X are `gemm_kernel` with op(A) = A / A^T, 2 m n l flops and one pass over A each).
GROUPS = {"a_pass": ("gemm_ax", "gemm_atx")}
# Single-workgroup kernels on the serial path (a chain of dependent pivots / rotation rounds): bounded by latency,
# not by a flop or byte rate; reported as time (and sweeps) only.
LATENCY_BOUND = ("cholesky", "jacobi", "small")


def measured_traffic(workload, kernel):
    """HBM bytes per launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summaries under profiles/ (each holds a
    line `traffic-json: {...}` keyed by workload and kernel class), or None when no counter run backs the pair."""
    import glob
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*hbm_counters*.md"))):
        for line in open(path):
            if line.startswith("traffic-json:"):
                try:
                    table = json.loads(line[len("traffic-json:"):])
                except ValueError:
                    continue
                if workload in table and kernel in table[workload]:
                    return float(table[workload][kernel])
    return None


def launch_model(name, cfg):
    """Algorithmic flops and bytes of ONE launch of a kernel class (every operand counted once), or None."""
    m, n, l, k, q = cfg.m, cfg.n, cfg.l, cfg.k, cfg.q
    sz = 4 if cfg.dtype == "f32" else 8
    if name in ("a_pass", "gemm_ax", "gemm_atx"):
        # read A once, read the skinny operand, write the result
        return dict(flops=2.0 * m * n * l, bytes=(m * n + n * l + m * l) * sz, mfma=cfg.dtype)
    # classes whose launches alternate between m-row and n-row panels: q + 1 CholeskyQR passes on each side,
    # the average launch is priced
    rows = (m + n) / 2.0
    if name == "gram":
        return dict(flops=2.0 * rows * l * l, bytes=rows * l * sz + l * l * 8, mfma="f64")
    if name == "apply_rinv":
        return dict(flops=2.0 * rows * l * l, bytes=2 * rows * l * sz + l * l * sz, mfma=cfg.dtype)
    if name == "lift":
        return dict(flops=2.0 * rows * l * k, bytes=rows * (l + k) * sz, mfma=cfg.dtype)
    if name == "sketch":
        return dict(flops=None, bytes=n * l * sz)
    return None


def roofline_for(name, avg_ms, cfg):
    """Position of one launch of `name` (average duration avg_ms) against the roofline that bounds it."""
    mod = launch_model(name, cfg)
    if mod is None or avg_ms <= 0:
        return None
    t = avg_ms * 1e-3
    t_mem = mod["bytes"] / PEAK_HBM
    flops = mod.get("flops")
    if "mfma" in mod and flops and flops / PEAK_MFMA[mod["mfma"]] > t_mem:
        peak = PEAK_MFMA[mod["mfma"]]
        return dict(bound="mfma", achieved=flops / t / 1e12, peak=peak / 1e12, unit="TFLOP/s",
                    frac=flops / t / peak, traffic=None, kernel=name, avg_us=avg_ms * 1e3)
    return dict(bound="hbm", achieved=mod["bytes"] / t / 1e9, peak=PEAK_HBM / 1e9, unit="GB/s",
                frac=mod["bytes"] / t / PEAK_HBM, traffic=None, kernel=name, avg_us=avg_ms * 1e3)


def grouped(kernels):
    """Per-class timings with the classes of GROUPS merged (launch-weighted)."""
    out = dict(kernels)
    for gname, members in GROUPS.items():
        have = [kernels[x] for x in members if x in kernels]
        if not have:
            continue
        for x in members:
            out.pop(x, None)
        ms = sum(h["ms_per_call"] for h in have)
        cnt = sum(h["launches_per_call"] for h in have)
        out[gname] = dict(ms_per_call=ms, launches_per_call=cnt, avg_us=ms / cnt * 1e3)
    return out


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
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
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
        (4000, 1000, 100, 28, 1, torch.float64, (1, 4, 32)),      # l = 128 in fp64: rotations accumulated in the workspace
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


def measure(ctx, cfg, A, steps, warmup, centered=False, with_graph=False, calibrate_copy=False):
    """Time `steps` full rsvd_run calls on A (resident in HBM), then the same steps again with HIP events around
    every kernel launch.  Returns wall time per call, its spread, the per-class kernel times and the diagnostics."""
    import numpy as np
    import torch
    from paper_2110_03423_amd import F32, F64

    dev = A.device
    dt = F32 if cfg.dtype == "f32" else F64
    ws = ctx.workspace(dt, cfg.m, cfg.n, cfg.k, cfg.p)
    out = (torch.empty(cfg.k, dtype=A.dtype, device=dev), torch.empty((cfg.m, cfg.k), dtype=A.dtype, device=dev),
           torch.empty((cfg.k, cfg.n), dtype=A.dtype, device=dev))
    mean_buf = torch.empty(cfg.n, dtype=A.dtype, device=dev)

    def step():
        ctx.rsvd_run(A, cfg.k, cfg.p, cfg.q, seed=cfg.seed, workspace=ws, want_info=False, out=out,
                     _mean=mean_buf if centered else None)

    for _ in range(warmup):
        step()
    if calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    _, _, _, info = ctx.rsvd_run(A, cfg.k, cfg.p, cfg.q, seed=cfg.seed, workspace=ws, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    res = dict(ms_per_step=(time.perf_counter() - t0) * 1e3 / steps, info=info)

    # per-call spread (paper's protocol: mean and standard deviation over repeated runs)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
    for a, b in evs:
        a.record(); step(); b.record()
    torch.cuda.synchronize()
    per_call = np.array([a.elapsed_time(b) for a, b in evs])
    res["mean_std_10"] = [round(float(per_call.mean()), 4), round(float(per_call.std()), 4)]

    if with_graph:
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
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        res["graph_ms"] = (time.perf_counter() - t0) * 1e3 / steps
        del graph

    # second pass over the same steps with HIP events around every kernel launch (recorded by the library on the
    # stream it launches on)
    ctx.rsvd_profile_enable(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    prof = ctx.rsvd_profile_read()
    ctx.rsvd_profile_enable(False)
    res["kernels"] = {name: dict(ms_per_call=tot / steps, launches_per_call=cnt / steps, avg_us=tot / cnt * 1e3)
                      for name, (tot, cnt) in prof.items()}
    return res


def dominant_roofline(cfg, kernels, info):
    """The kernel (classes of one template grouped) with the largest share of the call, and where it sits against
    its roofline.  A latency-bound class has no rate to quote: its entry carries time and sweeps instead."""
    g = grouped(kernels)
    name = max(g, key=lambda x: g[x]["ms_per_call"])
    roof = roofline_for(name, g[name]["avg_us"] * 1e-3, cfg)
    if roof is None:
        roof = dict(bound="latency", achieved=None, peak=None, unit=None, frac=None, traffic=None, kernel=name,
                    avg_us=g[name]["avg_us"], ms_per_call=g[name]["ms_per_call"], jacobi_sweeps=info.jacobi_sweeps)
    else:
        roof["traffic"] = measured_traffic(cfg.name, name)
    roof["share_of_call"] = g[name]["ms_per_call"] / sum(v["ms_per_call"] for v in g.values())
    return roof


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5,
                    help="benchmark configuration 1..5 (default 5: fp32 65536 x 16384, l = 576, the largest one)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the short runs of the other four configurations (extra key `other_configs`)")
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

    import torch
    import workloads
    from paper_2110_03423_amd import Rsvd

    if args.sweep:
        sweep(args)
        return
    if args.batched:
        batched(args)
        return
    cfg = workloads.CONFIGS[args.config]
    dev = "cuda:0"
    ctx = Rsvd(0)
    A = workloads.build(cfg, device=dev)
    res = measure(ctx, cfg, A, args.steps, args.warmup, centered=args.centered, with_graph=True,
                  calibrate_copy=args.calibrate_copy)
    info, kernels = res["info"], res["kernels"]
    roof = dominant_roofline(cfg, kernels, info)
    stage_roof = {}
    for name, v in grouped(kernels).items():
        r = roofline_for(name, v["avg_us"] * 1e-3, cfg)
        if r is not None:
            stage_roof[name] = dict(bound=r["bound"], achieved=round(r["achieved"], 3), unit=r["unit"],
                                    frac=round(r["frac"], 4), avg_us=round(v["avg_us"], 2))
        elif name in LATENCY_BOUND:
            stage_roof[name] = dict(bound="latency", ms_per_call=round(v["ms_per_call"], 4),
                                    launches_per_call=round(v["launches_per_call"], 1))

    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(cfg, A.cpu().numpy())
    del A
    torch.cuda.empty_cache()

    # the other configurations, shorter: wall time per call and the dominant kernel's position
    others = {}
    if not args.no_others and not args.centered:
        for cid, oc in workloads.CONFIGS.items():
            if cid == args.config:
                continue
            Ao = workloads.build(oc, device=dev)
            r = measure(ctx, oc, Ao, steps=10 if oc.m * oc.n > 1 << 27 else 20, warmup=2)
            d = dominant_roofline(oc, r["kernels"], r["info"])
            others[oc.name] = dict(dtype=oc.dtype, k=oc.k, p=oc.p, q=oc.q, ms_per_step=round(r["ms_per_step"], 4),
                                   mean_std_10=r["mean_std_10"], jacobi_sweeps=r["info"].jacobi_sweeps,
                                   dominant=d["kernel"], bound=d["bound"],
                                   frac=None if d["frac"] is None else round(d["frac"], 4),
                                   share_of_call=round(d["share_of_call"], 3))
            del Ao
            torch.cuda.empty_cache()

    ms_per_step = res["ms_per_step"]
    line = {
        "metric": "rsvd_wall_time_ms",
        "value": round(ms_per_step, 4),
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_mean_std_10": res["mean_std_10"],
        "ms_per_step_graph_replay": round(res["graph_ms"], 4),
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
        "other_configs": others,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
