#!/usr/bin/env python3
"""Benchmark of the PSO-PS synchronization step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one whole synchronization stage (selection + fused update) of the
named swarm, whose state is resident in HBM before the timed region starts.
Prints ONE JSON line: whole-job particle-parameters per second, the HBM
roofline of the update kernel measured live with events on the launch stream,
and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak

# HBM bytes per update-kernel launch from rocprofv3 --pmc runs (FETCH_SIZE and
# WRITE_SIZE, each scaled by what the counter reads for a plain copy of known
# size), keyed by workload and by the hash of the kernel source they were taken
# with: a changed kernel reports null until the counters are taken again.
MEASURED_TRAFFIC = {
    # profiles/update_kernel_resnet50x32_hbm_traffic.md: mean of three timed launches
    ("resnet50x32", "75be0b27336ea88a"): 16460299000.0,
}


def kernel_source_hash() -> str:
    """Hash of the code (comments and blank lines dropped) of every file under
    csrc/: kernels, their headers, the host launch code."""
    from paper_2009_03816_amd import build
    csrc = os.path.dirname(build.SOURCE)
    digest = hashlib.sha256()
    for name in sorted(os.listdir(csrc)):
        with open(os.path.join(csrc, name), "r") as f:
            code = [line.split("//")[0].rstrip() for line in f]
        digest.update((name + "\0" + "\n".join(t for t in code if t.strip())).encode())
    return digest.hexdigest()[:16]


def cpu_baseline(cfg, seconds_target: float = 15.0, all_cores: bool = True):
    """The oracle as it stands, single-threaded, on the first columns of the
    same swarm: one stage, sized for roughly `seconds_target` of CPU work."""
    import numpy as np
    from oracle import pso_ps_oracle as oracle
    from paper_2009_03816_amd import workloads as wl

    oracle.build()
    # size the sample from a short calibration pass of the same routine
    nc = 1 << 15
    cal = [np.zeros((cfg.K, nc), np.float32) for _ in range(3)]
    for _ in range(2):                                   # the first pass pays the page faults
        t0 = time.perf_counter()
        oracle.sync(cal[0], cal[1], cal[2], np.zeros(cfg.K, np.float32),
                    np.ones(cfg.K, np.float32), np.empty(nc, np.float32), np.float32(0.5),
                    np.float32(1.0), np.float32(1.0), 0, 0)
        rate = cfg.K * nc / (time.perf_counter() - t0)
    n = int(min(cfg.D, max(1024, seconds_target * rate / cfg.K)))
    n -= n % 2
    stages = int(max(1, min(4, round(seconds_target * rate / (cfg.K * n)))))
    rng = np.random.default_rng(cfg.seed)
    losses = wl.draw_losses(cfg, rng, stages + 1)
    x = (rng.standard_normal((cfg.K, n), dtype=np.float32) * np.float32(cfg.x_sigma))
    v = (rng.standard_normal((cfg.K, n), dtype=np.float32) * np.float32(cfg.v_sigma))
    pbest = x.copy()
    pbest_loss = np.minimum(losses[0], np.float32(3.0))  # about half of the particles improve
    gbest = np.empty(n, np.float32)
    pristine = [a.copy() for a in (x, v, pbest, pbest_loss)] if all_cores else None
    t0 = time.perf_counter()
    for s in range(stages):
        oracle.sync(x, v, pbest, pbest_loss, losses[s + 1], gbest, np.float32(cfg.w[0]),
                    np.float32(cfg.c1), np.float32(cfg.c2), cfg.seed, s)
    dt = time.perf_counter() - t0
    out = {"value": stages * cfg.K * n / dt, "unit": "particle-params/s", "cores": 1,
           "kind": "oracle",
           "sample": f"{stages} stage(s), K={cfg.K} x first {n} of {cfg.D} columns of {cfg.name}, "
                     f"{dt:.1f} s single-threaded"}
    if all_cores:
        # The same oracle call on disjoint column ranges, one thread each (ctypes
        # releases the GIL).  The random numbers are indexed by the column, so the
        # result must be the single-threaded one bit for bit.
        from concurrent.futures import ThreadPoolExecutor
        threads = max(1, min(16, len(os.sched_getaffinity(0))))
        x2, v2, p2, pl2 = pristine
        g2 = np.empty(n, np.float32)
        bounds = [n * t // threads for t in range(threads + 1)]

        def work(t, s):
            lo, hi = bounds[t], bounds[t + 1]
            if hi > lo:
                oracle.sync(x2[:, lo:hi], v2[:, lo:hi], p2[:, lo:hi], pl2.copy(), losses[s + 1],
                            g2[lo:hi], np.float32(cfg.w[0]), np.float32(cfg.c1), np.float32(cfg.c2),
                            cfg.seed, s, d0=lo)

        t0 = time.perf_counter()
        with ThreadPoolExecutor(threads) as pool:
            for s in range(stages):
                list(pool.map(lambda t: work(t, s), range(threads)))
                np.minimum(pl2, np.where(np.isnan(losses[s + 1]), np.inf, losses[s + 1]), out=pl2)
        dt2 = time.perf_counter() - t0
        same = all(np.array_equal(a.view(np.uint32), b.view(np.uint32))
                   for a, b in ((x, x2), (v, v2), (pbest, p2), (gbest, g2), (pbest_loss, pl2)))
        if not same:
            raise AssertionError("threaded oracle run differs from the single-threaded one")
        out["all_cores"] = {"value": stages * cfg.K * n / dt2, "cores": threads,
                            "bit_identical_to_one_core": True,
                            "sample": f"same sample, {dt2:.1f} s on {threads} threads"}
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="resnet50x32")
    ap.add_argument("--block", type=int, default=0, help="threads per workgroup (0 = default)")
    ap.add_argument("--super-tiles", type=int, default=0)
    ap.add_argument("--chunk-tiles", type=int, default=0)
    ap.add_argument("--wgs-per-cu", type=int, default=0)
    ap.add_argument("--variant", default="sync", choices=["sync", "history", "rows", "segments", "average"],
                    help="sync: the stage (default, the headline); history: historical gBest; "
                         "rows: K separate per-worker arrays; segments: one [K, n] array per "
                         "parameter tensor (needs a workload with a segment list); "
                         "average: parameter averaging")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch one plain device copy of 1 GiB (counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on ONE GPU (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2009_03816_amd as pso
    from paper_2009_03816_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    cfg = wl.CONFIGS[args.workload]
    K, D = cfg.K, cfg.D
    dev = torch.device("cuda:0")
    total = args.warmup + args.steps

    sw = wl.make_swarm(cfg, steps=total)
    if args.variant == "rows":                           # K separately allocated arrays
        xr = [torch.from_numpy(sw.x[i]).to(dev) for i in range(K)]
        vr = [torch.from_numpy(sw.v[i]).to(dev) for i in range(K)]
        pr = [t.clone() for t in xr]
        dx = xr[0]
    elif args.variant == "segments":                     # one dense [K, n] array per tensor
        if not cfg.segments:
            print(f"bench.py: workload {cfg.name} has no segment list", file=sys.stderr)
            return 2
        xs = [torch.from_numpy(a).to(dev) for a in wl.segment_views(sw.x, cfg.segments)]
        vs = [torch.from_numpy(a).to(dev) for a in wl.segment_views(sw.v, cfg.segments)]
        ps = [t.clone() for t in xs]
        gs = [torch.zeros(n, dtype=torch.float32, device=dev) for n in cfg.segments]
        dx = max(xs, key=lambda t: t.numel())
    else:
        dx = torch.from_numpy(sw.x).to(dev)
        dv = torch.from_numpy(sw.v).to(dev)
        dp = dx.clone()
    dpl = torch.from_numpy(sw.pbest_loss).to(dev)
    dloss = torch.from_numpy(sw.losses).to(dev)          # [total, K], resident
    dg = torch.zeros(D, dtype=torch.float32, device=dev)
    dgl = torch.full((1,), float("inf"), dtype=torch.float32, device=dev)
    w_tab, c1, c2 = [float(t) for t in sw.w], float(sw.c1), float(sw.c2)
    del sw

    h = pso.pso_ps_create(K, D, D, seg_sizes=list(cfg.segments)) if args.variant == "segments" \
        else pso.pso_ps_create(K, D)
    if args.block or args.super_tiles or args.chunk_tiles or args.wgs_per_cu:
        pso.pso_ps_set_launch(h, args.block, args.super_tiles, args.chunk_tiles, args.wgs_per_cu,
                              False)
    stream = torch.cuda.current_stream()

    def stage(s, ev=None):
        # events bracket the dominant kernel where the entry points allow it,
        # else the whole call (history, rows: selection + update)
        if args.variant == "sync":
            pso.pso_ps_select(h, dx, dpl, dloss[s], dg, stream)
        if ev:
            ev[0].record(stream)
        if args.variant == "sync":
            pso.pso_ps_update(h, dx, dv, dp, dg, w_tab[s], c1, c2, cfg.seed, s, stream)
        elif args.variant == "history":
            pso.pso_ps_sync_history(h, dx, dv, dp, dpl, dloss[s], dg, dgl, w_tab[s], c1, c2,
                                    cfg.seed, s, stream)
        elif args.variant == "rows":
            pso.pso_ps_sync_rows(h, xr, vr, pr, dpl, dloss[s], dg, w_tab[s], c1, c2, cfg.seed, s,
                                 stream)
        elif args.variant == "segments":
            pso.pso_ps_sync_segments(h, xs, vs, ps, dpl, dloss[s], gs, w_tab[s], c1, c2,
                                     cfg.seed, s, stream)
        else:
            pso.pso_ps_average(h, dx, dg, stream)
        if ev:
            ev[1].record(stream)

    for s in range(args.warmup):
        stage(s)
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        stage(args.warmup + k, events[k])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    kernel_ms = [a.elapsed_time(b) for a, b in events]
    avg_ms = sum(kernel_ms) / len(kernel_ms)
    median_ms = sorted(kernel_ms)[len(kernel_ms) // 2]
    if args.variant == "average":
        algo_bytes = 4.0 * D * (2 * K + 1)               # read K rows, write K rows and the mean
        kernel = "mean_kernel + broadcast_kernel"
    elif args.variant == "sync":
        algo_bytes = 4.0 * D * (5 * K + 1)               # per update launch
        kernel = "update_kernel"
    else:
        algo_bytes = 4.0 * D * (5 * K + 3)               # whole call: + read x_g, write gbest
        kernel = {"rows": "select_gbest_kernel + update_rows_kernel",
                  "segments": "select_gbest_segments_kernel + update_segments_kernel",
                  "history": "select_gbest_kernel + update_kernel"}[args.variant]
    achieved = algo_bytes / (avg_ms * 1e-3) / 1e9
    assert bool(torch.isfinite(dx).all()), "state went non-finite"

    # context for the roofline fraction: what a plain device copy of one [K, D]
    # array reaches on this machine, measured the same way (read + write bytes)
    if args.variant == "rows":
        copy_src, copy_dst = torch.stack(xr), torch.empty(K, D, dtype=torch.float32, device=dev)
    elif args.variant == "segments":
        copy_src = torch.cat([t.reshape(-1) for t in xs])
        copy_dst = torch.empty_like(copy_src)
    else:
        copy_src, copy_dst = dx, torch.empty_like(dx)
    copy_dst.copy_(copy_src)
    ce = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ce[0].record(stream)
    for _ in range(5):
        copy_dst.copy_(copy_src)
    ce[1].record(stream)
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * 4.0 * K * D / (ce[0].elapsed_time(ce[1]) * 1e-3) / 1e9
    del copy_src, copy_dst

    if args.copy_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    traffic = MEASURED_TRAFFIC.get((cfg.name, kernel_source_hash())) if args.variant == "sync" \
        else None
    out = {
        "metric": "PSO sync particle-params/s" if args.variant != "average"
        else "parameter-averaging particle-params/s", "value": K * D * args.steps / elapsed,
        "unit": "particle-params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: K={K} particles x D={D} fp32 parameters, "
                               f"w={cfg.w[0]}, c1={cfg.c1}, c2={cfg.c2}", "K": K, "D": D,
                   "variant": args.variant},
        "roofline": {"bound": "hbm", "kernel": kernel, "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "algorithmic_bytes_per_launch": algo_bytes,
                     "kernel_ms_avg": avg_ms, "kernel_ms_median": median_ms,
                     "kernel_ms_min": min(kernel_ms),
                     "device_copy_GBps_same_box": copy_gbs},
    }
    torch.cuda.synchronize()
    pso.pso_ps_destroy(h)
    del dx, dg
    if not args.no_cpu_baseline and args.variant == "sync":
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
