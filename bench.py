#!/usr/bin/env python3
"""Benchmark of the PSO-PS synchronization step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one whole synchronization stage (selection + fused update) of the
named swarm, whose state is resident in HBM before the timed region starts.
Prints ONE JSON line: whole-job particle-parameters per second over the timed
pso_ps_sync calls, the HBM roofline of the whole stage and of each of its two
kernels measured live with events on the launch stream, and the CPU oracle
timed on a bounded sample of the same workload.
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
    # profiles/update_others_kernel_resnet50x32_hbm_traffic.md: update_others_kernel, mean of the
    # three timed launches
    ("resnet50x32", "682a378094ddd28a"): 16153050000.0,
}

# What arithmetic-free streams over the same kind of arrays reached on one MI355X
# (profiles/ceilings_and_rejected_variants_resnet50x32.md, the best of each mix): the
# practical ceilings under the 8 TB/s peak.  Stored figures of another run; the in-place
# stream is also measured live on this run's own arrays (roofline.stream_ceiling.same_box).
STREAM_CEILING = {
    "in_place_3_reads_2_writes_GBps": 6400.0, "read_only_GBps": 7360.0, "copy_1r1w_GBps": 6630.0,
    "source": "profiles/ceilings_and_rejected_variants_resnet50x32.md (stored figures, another run)"}


def same_box_ceiling(torch, x, v, p, K, D, ld, stream):
    """The in-place 3-reads-2-writes stream of the probes library over this run's own x, v,
    pbest (written back unchanged), in the update pass's launch shape: GB/s, or None if the
    probes library is missing or the arrays are not 16-byte aligned."""
    try:
        from paper_2009_03816_amd import probes
        probes.load()
    except Exception:
        return None
    if any(t.data_ptr() % 16 for t in (x, v, p)) or (K > 1 and ld % 4):
        return None
    sink = torch.zeros(1, dtype=torch.float32, device=x.device)
    shape = dict(block_threads=64, quads=1, rows_per_wg=1, chunked=True, super_tiles=2048,
                 chunk_tiles=256, wgs_per_cu=20, nt_loads=True, nt_stores=True)
    run = lambda: probes.pso_ps_probe_stream("inplace", x, v, p, sink, K, D, ld,
                                             stream=int(stream.cuda_stream), **shape)
    for _ in range(2):
        run()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    marks[0].record(stream)
    for _ in range(10):
        run()
    marks[1].record(stream)
    torch.cuda.synchronize()
    return 10 * 20.0 * K * D / (marks[0].elapsed_time(marks[1]) * 1e-3) / 1e9


def kernel_source_hash() -> str:
    """Hash of the code (comments and blank lines dropped) of the stage's
    kernels, their header and the host launch code."""
    from paper_2009_03816_amd import build
    csrc = os.path.dirname(build.SOURCE)
    digest = hashlib.sha256()
    for name in ("pso_ps.hip", "tile_order.h"):
        with open(os.path.join(csrc, name), "r") as f:
            code = [line.split("//")[0].rstrip() for line in f]
        digest.update((name + "\0" + "\n".join(t for t in code if t.strip())).encode())
    return digest.hexdigest()[:16]


def stream_probe(args) -> int:
    """--variant stream: one arithmetic-free stream over the arrays of the
    workload (the probes library), timed like a stage."""
    import torch
    from paper_2009_03816_amd import probes
    from paper_2009_03816_amd import workloads as wl

    cfg = wl.CONFIGS[args.workload]
    K, D = cfg.K, cfg.D
    ld = args.ld or D
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg.seed)
    x, v, p = (torch.empty(K, ld, dtype=torch.float32, device=dev).normal_(0.0, cfg.x_sigma, generator=gen)
               for _ in range(3))
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    keep = x[:, :4096].clone()
    stream = torch.cuda.current_stream()
    # defaults: the launch shape of the update pass (64 threads, runs of 256 KiB, super-chunks
    # of 2 MiB, about 20 wavefronts per compute unit)
    block = args.block or 64
    tile_bytes = block * 16 * args.probe_quads
    shape = dict(block_threads=block, quads=args.probe_quads,
                 rows_per_wg=args.probe_rows_per_wg, chunked=args.probe_order == "chunked",
                 super_tiles=args.super_tiles or (2 << 20) // tile_bytes,
                 chunk_tiles=args.chunk_tiles or (256 << 10) // tile_bytes,
                 wgs_per_cu=args.wgs_per_cu or max(3, 20 * 64 // block),
                 nt_loads=bool(args.probe_nt_loads),
                 nt_stores=bool(args.probe_nt_stores),
                 absolute_chunks=args.probe_absolute_chunks)

    kernel_name = "stream_kernel"
    if args.probe_policy:
        # the in-place mix in its default shape with explicit cache-policy bits
        loads, stores = (probes.policy_bits(t) for t in args.probe_policy.split(","))
        assert args.probe_mix == "inplace" and block == 64 and args.probe_quads == 1
        shape = dict(super_tiles=shape["super_tiles"], chunk_tiles=shape["chunk_tiles"],
                     wgs_per_cu=shape["wgs_per_cu"], load_policy=loads, store_policy=stores)
        kernel_name = "policy_kernel"

    def stage(_):
        if args.probe_policy:
            probes.pso_ps_probe_policy(x, v, p, sink, K, D, ld, stream=int(stream.cuda_stream),
                                       **shape)
        else:
            probes.pso_ps_probe_stream(args.probe_mix, x, v, p, sink, K, D, ld,
                                       stream=int(stream.cuda_stream), **shape)

    for s in range(args.warmup):
        stage(s)
    elapsed, ms = time_stages(stage, 0, args.steps, stream, torch)
    t = summary(ms)
    if args.probe_mix != "copy":
        assert torch.equal(x[:, :4096], keep), "the probe changed the arrays"
    floats = {"read": 3, "copy": 2, "inplace": 5}[args.probe_mix]
    nbytes = 4.0 * K * D * floats
    gbs = nbytes / (t["avg"] * 1e-3) / 1e9
    print(json.dumps({
        "metric": "stream probe GB/s", "value": gbs, "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: K={K} x D={D} fp32, row stride {ld}",
                   "variant": "stream", "mix": args.probe_mix, **shape},
        "roofline": {"bound": "hbm", "kernel": kernel_name, "achieved": gbs,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                     "traffic": None, "algorithmic_bytes_per_launch": nbytes,
                     "kernel_ms_avg": t["avg"], "kernel_ms_median": t["median"],
                     "kernel_ms_min": t["min"]}}))
    return 0


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


def time_stages(stage, first, count, stream, torch, per_stage_events=True):
    """Enqueue `count` stages, wait once, and return (wall seconds, per-stage
    milliseconds).  With per_stage_events an event is recorded after every
    stage; without, only before the first and after the last (nothing but the
    stages' own kernels sits in the stream) and every stage is given the mean."""
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(count + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record(stream)
    for k in range(count):
        stage(first + k)
        if per_stage_events or k == count - 1:
            marks[k + 1].record(stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    if not per_stage_events:
        return elapsed, [marks[0].elapsed_time(marks[count]) / count] * count
    return elapsed, [marks[k].elapsed_time(marks[k + 1]) for k in range(count)]


def summary(ms):
    return {"avg": sum(ms) / len(ms), "median": sorted(ms)[len(ms) // 2], "min": min(ms)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="resnet50x32",
                    help="a named configuration, or KxD (e.g. 8x250000) for a swarm of that shape")
    ap.add_argument("--block", type=int, default=0, help="threads per workgroup (0 = default)")
    ap.add_argument("--super-tiles", type=int, default=0)
    ap.add_argument("--chunk-tiles", type=int, default=0)
    ap.add_argument("--wgs-per-cu", type=int, default=0)
    ap.add_argument("--force-generic", action="store_true",
                    help="element-wise path instead of the 128-bit one (a measurement of that path)")
    ap.add_argument("--fused-rows", type=int, default=0,
                    help="sync, history: the single-pass kernels with this many rows in flight per "
                         "workgroup (pso_ps_set_variant) instead of the default two kernels")
    ap.add_argument("--best-first", type=int, default=-1,
                    help="0: the copy-based split of the stage (selection + gbest copy, then all K "
                         "particles) instead of the default (selection + the best particle, then "
                         "the others)")
    ap.add_argument("--single-launch", type=int, default=-1,
                    help="pso_ps_set_single_launch: 1 the whole stage as one launch (K <= 64), 0 "
                         "never, -1 (default) the library's choice: small swarms only")
    ap.add_argument("--chunk-origin", type=int, default=-1,
                    help="pso_ps_set_variant's chunk_origin (default: the library's)")
    ap.add_argument("--ld", type=int, default=0,
                    help="row stride in elements (default D, the dense layout of the metric)")
    ap.add_argument("--misalign", default="",
                    help="four element offsets 'x,v,pbest,gbest' of the arrays inside their "
                         "allocations (default: all 0, i.e. 16-byte aligned and congruent)")
    ap.add_argument("--variant", default="sync",
                    choices=["sync", "history", "rows", "segments", "average", "stream"],
                    help="sync: the stage (default, the headline); history: historical gBest; "
                         "rows: K separate per-worker arrays; segments: one [K, n] array per "
                         "parameter tensor (needs a workload with a segment list); "
                         "average: parameter averaging; stream: an arithmetic-free stream over "
                         "the same arrays (the --probe-* options), a measured ceiling")
    ap.add_argument("--probe-mix", default="inplace", choices=["read", "copy", "inplace"],
                    help="stream: read x, v, pbest / copy x to v / read all three and write x, v back")
    ap.add_argument("--probe-order", default="chunked", choices=["plain", "chunked"])
    ap.add_argument("--probe-rows-per-wg", type=int, default=1)
    ap.add_argument("--probe-quads", type=int, default=1)
    ap.add_argument("--probe-nt-loads", type=int, default=1)
    ap.add_argument("--probe-nt-stores", type=int, default=1)
    ap.add_argument("--probe-absolute-chunks", type=int, default=0)
    ap.add_argument("--probe-policy", default="",
                    help="--variant stream: LOADS,STORES cache-policy bits for the in-place mix in "
                         "its default shape, each a sum of sc0, nt, sc1 or none (e.g. nt,nt+sc1)")
    ap.add_argument("--graph", action="store_true",
                    help="also capture 100 stages into a HIP graph, replay it and report the time "
                         "per stage (roofline.stage.hip_graph_replay_ms)")
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
    if args.variant == "stream":
        return stream_probe(args)
    if "x" in args.workload and args.workload.replace("x", "").isdigit():
        # "KxD": a swarm of that shape with resnet20's value distributions (for size sweeps)
        k_arg, d_arg = (int(t) for t in args.workload.split("x"))
        cfg = wl.SwarmConfig(**{**wl.CONFIGS["resnet20"].__dict__, "name": args.workload,
                                "K": k_arg, "D": d_arg})
    else:
        cfg = wl.CONFIGS[args.workload]
    K, D = cfg.K, cfg.D
    dev = torch.device("cuda:0")
    total = args.warmup + 3 * args.steps            # the timed pass, the per-kernel pass and
                                                     # the pass with an event after every stage
    offs = [int(t) for t in args.misalign.split(",")] if args.misalign else [0, 0, 0, 0]

    def shifted(a, off):
        """`a` on the device, starting `off` elements into its allocation."""
        flat = torch.empty(a.size + off, dtype=torch.float32, device=dev)
        view = flat[off:].view(a.shape)
        view.copy_(torch.from_numpy(a))
        return view

    ld = args.ld or D
    sw = wl.make_swarm(cfg, ld=ld, steps=total)
    if args.variant == "rows":                           # K separately allocated arrays
        xr = [shifted(sw.x[i], offs[0]) for i in range(K)]
        vr = [shifted(sw.v[i], offs[1]) for i in range(K)]
        pr = [shifted(sw.x[i], offs[2]) for i in range(K)]
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
        dx, dv, dp = shifted(sw.x, offs[0]), shifted(sw.v, offs[1]), shifted(sw.x, offs[2])
    dpl = torch.from_numpy(sw.pbest_loss).to(dev)
    dloss = torch.from_numpy(sw.losses).to(dev)          # [total, K], resident
    dg = shifted(np.zeros(D, np.float32), offs[3])
    dgl = torch.full((1,), float("inf"), dtype=torch.float32, device=dev)
    # the workload's inertia schedule covers cfg.steps stages; longer runs go round it again
    w_tab = [float(sw.w[s % cfg.steps]) for s in range(total)]
    c1, c2 = float(sw.c1), float(sw.c2)
    del sw

    h = pso.pso_ps_create(K, D, D, seg_sizes=list(cfg.segments)) if args.variant == "segments" \
        else pso.pso_ps_create(K, D, ld)
    if args.block or args.super_tiles or args.chunk_tiles or args.wgs_per_cu or args.force_generic:
        pso.pso_ps_set_launch(h, args.block, args.super_tiles, args.chunk_tiles, args.wgs_per_cu,
                              args.force_generic)
    if args.fused_rows or args.chunk_origin >= 0 or args.best_first >= 0:
        # (a chunk origin is an option of the copy-based split's update pass)
        best_first = args.best_first != 0 and args.chunk_origin < 0
        pso.pso_ps_set_variant(h, args.fused_rows, max(args.chunk_origin, 0), best_first)
    if args.single_launch >= 0:
        pso.pso_ps_set_single_launch(h, args.single_launch)
    stream = torch.cuda.current_stream()

    # host arrays of device pointers for the ragged and row-pointer calls, built once
    if args.variant == "rows":
        xr_t, vr_t, pr_t = (pso.pso_ps_pointer_table(t) for t in (xr, vr, pr))
    elif args.variant == "segments":
        xs_t, vs_t, ps_t, gs_t = (pso.pso_ps_pointer_table(t) for t in (xs, vs, ps, gs))

    def stage(s, st=None):
        """One whole synchronization stage through the entry point of the variant."""
        st = st or stream
        if args.variant == "sync":
            pso.pso_ps_sync(h, dx, dv, dp, dpl, dloss[s], dg, w_tab[s], c1, c2, cfg.seed, s, st)
        elif args.variant == "history":
            pso.pso_ps_sync_history(h, dx, dv, dp, dpl, dloss[s], dg, dgl, w_tab[s], c1, c2,
                                    cfg.seed, s, st)
        elif args.variant == "rows":
            pso.pso_ps_sync_rows(h, xr_t, vr_t, pr_t, dpl, dloss[s], dg, w_tab[s], c1, c2, cfg.seed,
                                 s, st)
        elif args.variant == "segments":
            pso.pso_ps_sync_segments(h, xs_t, vs_t, ps_t, dpl, dloss[s], gs_t, w_tab[s], c1, c2,
                                     cfg.seed, s, st)
        else:
            pso.pso_ps_average(h, dx, dg, st)

    # -- the timed region: K whole stages through the entry point ---------------------------
    for s in range(args.warmup):
        stage(s)
    elapsed, stage_ms = time_stages(stage, args.warmup, args.steps, stream, torch,
                                    per_stage_events=False)
    stage_t = summary(stage_ms)

    # -- a second pass over as many stages, split at the kernel boundary --------------------
    # (sync only: pso_ps_sync_begin + pso_ps_sync_finish are the two launches of pso_ps_sync,
    # bit for bit; an event between them gives each kernel's own duration on the launch stream)
    first_ms, second_ms = [], []
    split_pass = args.variant == "sync" and not args.fused_rows
    if split_pass:
        marks = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
        for k in range(args.steps):
            s = args.warmup + args.steps + k
            a = (h, dx, dv, dp, dpl, dloss[s], dg, w_tab[s], c1, c2, cfg.seed, s, stream)
            marks[k][0].record(stream)
            pso.pso_ps_sync_begin(*a)
            marks[k][1].record(stream)
            pso.pso_ps_sync_finish(*a)
            marks[k][2].record(stream)
        torch.cuda.synchronize()
        first_ms = [m[0].elapsed_time(m[1]) for m in marks]
        second_ms = [m[1].elapsed_time(m[2]) for m in marks]

    # -- a third pass with an event after every stage: the spread from stage to stage --------
    _, each_ms = time_stages(stage, args.warmup + 2 * args.steps, args.steps, stream, torch)
    each_t = summary(each_ms)
    assert bool(torch.isfinite(dx).all()), "state went non-finite"

    # -- optional: the same stages replayed from a HIP graph --------------------------------
    graph_ms = None
    if args.graph:
        per_graph = min(args.steps, 100)
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for k in range(per_graph):
                stage(args.warmup + k, side)
        graph.replay()
        torch.cuda.synchronize()
        replays = max(1, args.steps // per_graph)
        ge = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ge[0].record(stream)
        for _ in range(replays):
            graph.replay()
        ge[1].record(stream)
        torch.cuda.synchronize()
        graph_ms = ge[0].elapsed_time(ge[1]) / (replays * per_graph)

    # -- byte counts -------------------------------------------------------------------------
    if args.variant == "average":
        stage_bytes = 4.0 * D * (2 * K + 1)              # read K rows, write K rows and the mean
        kernel = "mean_kernel + broadcast_kernel"
    else:
        stage_bytes = 4.0 * D * (5 * K + 1)              # the least a stage can move (see below)
        kernel = {"sync": "update_others_kernel", "rows": "select_gbest_kernel + update_rows_kernel",
                  "segments": "select_gbest_segments_kernel + update_segments_kernel",
                  "history": "select_gbest_kernel + update_kernel"}[args.variant]
    stage_gbs = stage_bytes / (stage_t["avg"] * 1e-3) / 1e9
    fits_one = args.variant in ("sync", "history", "rows") or (
        args.variant == "segments" and sum(1 for n in cfg.segments if n > 0) <= 32)
    one_launch = fits_one and not args.fused_rows and (
        args.single_launch == 1 or (args.single_launch < 0 and K <= 16
                                    and K * D <= pso.PSO_PS_SINGLE_LAUNCH_MAX_PARAMS))
    stage_roof = {
        "launches": "one: whole_stage_kernel (the per-kernel pass below is the same stage taken "
                    "in two launches through pso_ps_sync_begin / pso_ps_sync_finish)"
        if one_launch else "two or more: see roofline.kernel",
        "what": "the whole entry-point call: one event before the first and one after the last "
                "of the timed stages, divided by their number",
        "bytes": stage_bytes, "ms_avg": stage_t["avg"],
        "per_stage_events": {"ms_avg": each_t["avg"], "ms_median": each_t["median"],
                             "ms_min": each_t["min"],
                             "what": "a further pass over as many later stages with an event "
                                     "after every stage"},
        "achieved": stage_gbs, "frac": stage_gbs / HBM_PEAK_GBS,
        "bytes_are": "algorithmic minimum 4*D*(5K+1): x, v read and written, pbest read or "
                     "written, gbest written once; the two kernels move 4*D*(5K+2), one more "
                     "pass over gbest"
        if args.variant != "average" else "4*D*(2K+1)"}

    # context for the fractions: torch's own device-to-device copy of one [K, D] array on
    # this box (read + write bytes).  It is NOT a ceiling: the library's kernels beat it.
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

    if args.fused_rows and args.variant in ("sync", "history"):
        kernel = "select_only_kernel + fused_rows_kernel"
    if split_pass:
        second, first = summary(second_ms), summary(first_ms)
        if args.best_first == 0 or args.chunk_origin >= 0:   # the copy-based split
            kernel, first_kernel = "update_kernel", "select_gbest_kernel"
            kernel_bytes = 4.0 * D * (5 * K + 1)         # K rows at 20 B + the first read of gbest
            first_bytes = 8.0 * D                        # read row g, write gbest
        else:                                            # the default: best particle first
            kernel, first_kernel = "update_others_kernel", "select_move_best_kernel"
            kernel_bytes = 4.0 * D * (5 * (K - 1) + 1)   # K-1 rows at 20 B + the first read of gbest
            first_bytes = 24.0 * D                       # row g at 20 B + the write of gbest
        achieved = kernel_bytes / (second["avg"] * 1e-3) / 1e9
        default_shape = not (args.block or args.super_tiles or args.chunk_tiles or args.wgs_per_cu
                             or args.force_generic or args.misalign or args.ld
                             or args.best_first >= 0 or args.chunk_origin >= 0)
        key = (cfg.name, kernel_source_hash())
        traffic = MEASURED_TRAFFIC.get(key) if default_shape else None
        roofline = {
            "bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
            "traffic_is": "a stored rocprofv3 --pmc reading (FETCH_SIZE + WRITE_SIZE, "
                          "profiles/update_others_kernel_resnet50x32_hbm_traffic.md), valid for the "
                          "kernel source hash it was taken with; null once the kernels have changed",
            "kernel_source_hash": key[1],
            "algorithmic_bytes_per_launch": kernel_bytes,
            "kernel_ms_avg": second["avg"], "kernel_ms_median": second["median"],
            "kernel_ms_min": second["min"],
            "kernel_pass": "a second pass over the same number of stages as pso_ps_sync_begin + "
                           "pso_ps_sync_finish with an event between the two kernels",
            "first_kernel": {"kernel": first_kernel, "bytes": first_bytes,
                             "ms_avg": first["avg"], "ms_median": first["median"],
                             "ms_min": first["min"],
                             "achieved": first_bytes / (first["avg"] * 1e-3) / 1e9,
                             "frac": first_bytes / (first["avg"] * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "stage": stage_roof,
        }
    else:
        roofline = {"bound": "hbm", "kernel": kernel, "achieved": stage_gbs, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": stage_gbs / HBM_PEAK_GBS, "traffic": None,
                    "algorithmic_bytes_per_launch": stage_bytes, "kernel_ms_avg": stage_t["avg"],
                    "kernel_ms_median": stage_t["median"], "kernel_ms_min": stage_t["min"],
                    "stage": stage_roof}
    roofline["stream_ceiling"] = dict(STREAM_CEILING)
    if args.variant in ("sync", "history"):
        live = same_box_ceiling(torch, dx, dv, dp, K, D, ld, stream)
        roofline["stream_ceiling"]["same_box"] = {
            "in_place_3_reads_2_writes_GBps": live,
            "what": "arithmetic-free stream over this run's x, v, pbest in the update pass's "
                    "launch shape, measured after the timed stages"}
    roofline["torch_copy_GBps_same_box"] = copy_gbs
    if graph_ms is not None:
        roofline["stage"]["hip_graph_replay_ms"] = graph_ms

    out = {
        "metric": "PSO sync particle-params/s" if args.variant != "average"
        else "parameter-averaging particle-params/s", "value": K * D * args.steps / elapsed,
        "unit": "particle-params/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: K={K} particles x D={D} fp32 parameters, "
                               f"w={cfg.w[0]}, c1={cfg.c1}, c2={cfg.c2}", "K": K, "D": D,
                   "variant": args.variant,
                   "entry_point": {"sync": "pso_ps_sync", "history": "pso_ps_sync_history",
                                   "rows": "pso_ps_sync_rows", "segments": "pso_ps_sync_segments",
                                   "average": "pso_ps_average"}[args.variant]},
        "roofline": roofline,
    }
    if args.force_generic or args.misalign or args.fused_rows or args.ld:
        out["config"]["path"] = ("element-wise (forced)" if args.force_generic else "128-bit") + \
            (f", array offsets {offs}" if args.misalign else "") + \
            (f", single pass with {args.fused_rows} rows in flight" if args.fused_rows else "") + \
            (f", row stride {ld}" if args.ld else "")
    torch.cuda.synchronize()
    pso.pso_ps_destroy(h)
    del dx, dg
    if not args.no_cpu_baseline and args.variant == "sync":
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
