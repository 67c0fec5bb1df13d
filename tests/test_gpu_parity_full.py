"""GPU parity at the full benchmark sizes, in the default launch shape.  The
oracle advances column windows (start, middle, end; the update of a column
never looks at another column) and every stage is compared there; over the
whole arrays the selection rules and Eq. (7) are checked as exact properties."""
import gc

import numpy as np
import pytest
import torch

import paper_2009_03816_amd as pso
from paper_2009_03816_amd import workloads as wl

import gpu_harness as gh

pytestmark = pytest.mark.gpu
F32 = np.float32


def windows_of(D):
    mid = D // 2 - 1501            # odd start: windows need not respect any tile or pair boundary
    return [(0, 3000), (mid, mid + 3001), (D - 3000, D)]


@pytest.mark.parametrize("name", ["vgg16", "resnet50x32"])
def test_full_size_config(oracle, name):
    cfg = wl.CONFIGS[name]
    K, D = cfg.K, cfg.D
    print(f"[case] full-size config {name}: K={K} D={D}", flush=True)
    sw = wl.make_swarm(cfg)
    wins = windows_of(D)
    host = [[np.ascontiguousarray(a[:, lo:hi]) for a in (sw.x, sw.v, sw.pbest)] for lo, hi in wins]
    hpl = [sw.pbest_loss.copy() for _ in wins]
    dx, dv = gh.to_dev(sw.x), gh.to_dev(sw.v)
    dp = dx.clone()                                  # initial personal best = position (Algorithm 2)
    dpl = gh.to_dev(sw.pbest_loss)
    dg = torch.zeros(D, dtype=torch.float32, device=gh.dev())
    losses, w_tab, c1, c2 = sw.losses, sw.w, float(sw.c1), float(sw.c2)
    del sw
    gc.collect()
    print("[case] swarm resident on the device", flush=True)
    h = pso.pso_ps_create(K, D)
    try:
        for s in range(cfg.steps):
            x_old, p_old = dx.clone(), dp.clone()
            w = float(w_tab[s])
            pso.pso_ps_sync(h, dx, dv, dp, dpl, gh.to_dev(losses[s]), dg, w, c1, c2, cfg.seed, s)
            g_dev, imp_dev = pso.pso_ps_last_selection(h, K)
            # oracle on the windows
            for (lo, hi), (hx, hv, hp), pl in zip(wins, host, hpl):
                hg = np.empty(hi - lo, F32)
                g, improved = oracle.sync(hx, hv, hp, pl, losses[s], hg, F32(w), F32(c1), F32(c2),
                                          cfg.seed, s, d0=lo)
                what = f"{name} step {s} columns [{lo},{hi})"
                assert g_dev == g and imp_dev == [bool(t) for t in improved], what
                gh.assert_bits_equal(dg[lo:hi].cpu().numpy(), hg, what + ": gbest")
                gh.assert_bits_equal(dp[:, lo:hi].cpu().numpy(), hp, what + ": pbest")
                gh.assert_close(dx[:, lo:hi].cpu().numpy(), hx, what + ": x")
                gh.assert_close(dv[:, lo:hi].cpu().numpy(), hv, what + ": v")
                gh.assert_bits_equal(dpl.cpu().numpy(), pl, what + ": pbest_loss")
            # whole arrays: Algorithm 3, Algorithm 1 and Eq. (7) as exact properties
            as_bits = lambda t: t.view(torch.int32)
            assert torch.equal(as_bits(dg), as_bits(x_old[g_dev])), "gbest != x_g before the move"
            for i in range(K):
                src = x_old[i] if imp_dev[i] else p_old[i]
                assert torch.equal(as_bits(dp[i]), as_bits(src)), f"pbest row {i}"
            assert torch.equal(dx, x_old + dv), "x' != x + v'"
            assert bool(torch.isfinite(dv).all())
            del x_old, p_old
            print(f"[case] {name} step {s} ok (g={g_dev}, improved={sum(imp_dev)})", flush=True)
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


def test_full_size_per_layer_layout(oracle):
    """The large swarm held as 161 per-tensor [K, n] arrays (six launches' worth
    of segments): windows of a small, a mid-sized, the largest and the last
    tensors against the oracle, every array against the flat call's properties."""
    cfg = wl.CONFIGS["resnet50x32_layers"]
    K, D, sizes = cfg.K, cfg.D, list(cfg.segments)
    print(f"[case] full-size per-layer layout: K={K} D={D} in {len(sizes)} tensors", flush=True)
    sw = wl.make_swarm(cfg, steps=3)
    starts = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    big = int(np.argmax(sizes))
    picks = [(0, 0, sizes[0]), (1, 0, sizes[1]), (3, 0, 3000), (big, 0, 2500),
             (big, sizes[big] // 2 - 999, sizes[big] // 2 + 1200), (big, sizes[big] - 2048, sizes[big]),
             (len(sizes) - 2, 1_000_001, 1_003_000), (len(sizes) - 1, 0, sizes[-1])]
    host = []
    for s, lo, hi in picks:
        a, b = starts[s] + lo, starts[s] + hi
        host.append([np.ascontiguousarray(t[:, a:b]) for t in (sw.x, sw.v, sw.pbest)])
    hpl = [sw.pbest_loss.copy() for _ in picks]
    xs = [torch.from_numpy(a).to(gh.dev()) for a in wl.segment_views(sw.x, sizes)]
    vs = [torch.from_numpy(a).to(gh.dev()) for a in wl.segment_views(sw.v, sizes)]
    ps = [t.clone() for t in xs]
    gs = [torch.zeros(n, dtype=torch.float32, device=gh.dev()) for n in sizes]
    dpl = gh.to_dev(sw.pbest_loss)
    losses, c1, c2 = sw.losses, float(sw.c1), float(sw.c2)
    w_tab = sw.w
    del sw
    gc.collect()
    h = pso.pso_ps_create(K, D, D, seg_sizes=sizes)
    try:
        for step in range(3):
            x_old = [t.clone() for t in xs]
            w = float(w_tab[step])
            pso.pso_ps_sync_segments(h, xs, vs, ps, dpl, gh.to_dev(losses[step]), gs, w, c1, c2,
                                     cfg.seed, step)
            g_dev, imp_dev = pso.pso_ps_last_selection(h, K)
            for (s, lo, hi), (hx, hv, hp), pl in zip(picks, host, hpl):
                hg = np.empty(hi - lo, F32)
                g, improved = oracle.sync(hx, hv, hp, pl, losses[step], hg, F32(w), F32(c1), F32(c2),
                                          cfg.seed, step, d0=int(starts[s]) + lo)
                what = f"per-layer step {step} tensor {s} columns [{lo},{hi})"
                assert g_dev == g and imp_dev == [bool(t) for t in improved], what
                gh.assert_bits_equal(gs[s][lo:hi].cpu().numpy(), hg, what + ": gbest")
                gh.assert_bits_equal(ps[s][:, lo:hi].cpu().numpy(), hp, what + ": pbest")
                gh.assert_close(xs[s][:, lo:hi].cpu().numpy(), hx, what + ": x")
                gh.assert_close(vs[s][:, lo:hi].cpu().numpy(), hv, what + ": v")
            for s in range(len(sizes)):
                assert torch.equal(gs[s].view(torch.int32), x_old[s][g_dev].view(torch.int32))
                assert torch.equal(xs[s], x_old[s] + vs[s]), f"tensor {s}: x' != x + v'"
            print(f"[case] per-layer step {step} ok (g={g_dev}, improved={sum(imp_dev)})", flush=True)
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


def test_full_size_variants(oracle):
    """Row-pointer mode, historical gBest and parameter averaging at the full
    benchmark size (K=32, D=25,557,032), each against the oracle on column
    windows, from one generated swarm."""
    cfg = wl.CONFIGS["resnet50x32"]
    K, D = cfg.K, cfg.D
    print(f"[case] full-size variants: K={K} D={D}", flush=True)
    sw = wl.make_swarm(cfg, steps=3)
    wins = windows_of(D)
    losses, c1, c2, w = sw.losses.copy(), float(sw.c1), float(sw.c2), float(sw.w[0])
    losses[2] = losses[:2].min() + F32(1.0)          # a stage that keeps the old gbest

    def window_state():
        return [[np.ascontiguousarray(a[:, lo:hi]) for a in (sw.x, sw.v, sw.pbest)]
                for lo, hi in wins], [sw.pbest_loss.copy() for _ in wins]

    # -- K separate row arrays ----------------------------------------------------------
    host, hpl = window_state()
    xr = [torch.from_numpy(sw.x[i]).to(gh.dev()) for i in range(K)]
    vr = [torch.from_numpy(sw.v[i]).to(gh.dev()) for i in range(K)]
    pr = [t.clone() for t in xr]
    dpl, dg = gh.to_dev(sw.pbest_loss), torch.zeros(D, dtype=torch.float32, device=gh.dev())
    h = pso.pso_ps_create(K, D)
    try:
        for step in range(2):
            pso.pso_ps_sync_rows(h, xr, vr, pr, dpl, gh.to_dev(losses[step]), dg, w, c1, c2,
                                 cfg.seed, step)
            g_dev, imp_dev = pso.pso_ps_last_selection(h, K)
            for (lo, hi), (hx, hv, hp), pl in zip(wins, host, hpl):
                hg = np.empty(hi - lo, F32)
                g, improved = oracle.sync(hx, hv, hp, pl, losses[step], hg, F32(w), F32(c1), F32(c2),
                                          cfg.seed, step, d0=lo)
                what = f"rows step {step} columns [{lo},{hi})"
                assert g_dev == g and imp_dev == [bool(t) for t in improved], what
                cut = lambda rows: torch.stack([t[lo:hi] for t in rows]).cpu().numpy()
                gh.assert_bits_equal(dg[lo:hi].cpu().numpy(), hg, what + ": gbest")
                gh.assert_bits_equal(cut(pr), hp, what + ": pbest")
                gh.assert_close(cut(xr), hx, what + ": x")
                gh.assert_close(cut(vr), hv, what + ": v")
            print(f"[case] rows step {step} ok", flush=True)
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)
    del xr, vr, pr
    gc.collect()

    # -- historical gBest on the stacked layout -----------------------------------------
    host, hpl = window_state()
    hgb = [np.zeros(hi - lo, F32) for lo, hi in wins]
    hgl = [np.array([np.inf], F32) for _ in wins]
    dx, dv = gh.to_dev(sw.x), gh.to_dev(sw.v)
    dp = dx.clone()
    dpl, dgl = gh.to_dev(sw.pbest_loss), gh.to_dev(np.array([np.inf], F32))
    dg.zero_()
    del sw
    gc.collect()
    h = pso.pso_ps_create(K, D)
    try:
        kept = 0
        for step in range(3):
            pso.pso_ps_sync_history(h, dx, dv, dp, dpl, gh.to_dev(losses[step]), dg, dgl, w, c1, c2,
                                    cfg.seed, step)
            g_dev, imp_dev, rep_dev = pso.pso_ps_last_selection(h, K, with_replaced=True)
            for (lo, hi), (hx, hv, hp), pl, hg, gl in zip(wins, host, hpl, hgb, hgl):
                g, improved, rep = oracle.sync(hx, hv, hp, pl, losses[step], hg, F32(w), F32(c1),
                                               F32(c2), cfg.seed, step, d0=lo, gbest_loss=gl)
                what = f"history step {step} columns [{lo},{hi})"
                assert (g_dev, imp_dev, rep_dev) == (g, [bool(t) for t in improved], rep), what
                gh.assert_bits_equal(dgl.cpu().numpy(), gl, what + ": gbest_loss")
                gh.assert_bits_equal(dg[lo:hi].cpu().numpy(), hg, what + ": gbest")
                gh.assert_bits_equal(dp[:, lo:hi].cpu().numpy(), hp, what + ": pbest")
                gh.assert_close(dx[:, lo:hi].cpu().numpy(), hx, what + ": x")
                gh.assert_close(dv[:, lo:hi].cpu().numpy(), hv, what + ": v")
            kept += not rep_dev
            print(f"[case] history step {step} ok (replaced={rep_dev})", flush=True)
        assert kept == 1

        # -- parameter averaging of the positions just produced -----------------------------
        dmean = torch.zeros(D, dtype=torch.float32, device=gh.dev())
        before = [dx[:, lo:hi].cpu().numpy() for lo, hi in wins]
        pso.pso_ps_average(h, dx, dmean)
        for (lo, hi), hx in zip(wins, before):
            hmean = np.empty(hi - lo, F32)
            oracle.average(hx, hmean)
            gh.assert_bits_equal(dmean[lo:hi].cpu().numpy(), hmean, f"mean columns [{lo},{hi})")
            gh.assert_bits_equal(dx[:, lo:hi].cpu().numpy(), hx, f"averaged rows [{lo},{hi})")
        assert all(torch.equal(dx[i].view(torch.int32), dmean.view(torch.int32)) for i in range(K))
        print("[case] averaging ok", flush=True)
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


def test_rows_longer_than_2_to_31_columns(oracle):
    """Maximum sizes: two rows of 2^31 + 5,242,886 columns each (8.6 GB per row),
    so that column indices, byte offsets and the flat coordinate of the random
    numbers all pass 32 bits.  Inputs are drawn on the device (seeded); the
    oracle advances windows at the start, across column 2^30 (byte offset 2^32),
    across column 2^31, and at the ragged end."""
    K, D = 2, (1 << 31) + 5 * (1 << 20) + 6
    seed, c1, c2, w = 11, 1.3, 1.6, 0.6
    print(f"[case] long rows: K={K} D={D}", flush=True)
    gen = torch.Generator(device=gh.dev())
    gen.manual_seed(2031)
    dx = torch.empty(K, D, dtype=torch.float32, device=gh.dev())
    dv = torch.empty(K, D, dtype=torch.float32, device=gh.dev())
    dx.normal_(0.0, 0.02, generator=gen)
    dv.normal_(0.0, 0.002, generator=gen)
    dp = dx.clone()
    dg = torch.zeros(D, dtype=torch.float32, device=gh.dev())
    wins = [(0, 2500), ((1 << 30) - 1501, (1 << 30) + 1500), ((1 << 31) - 1499, (1 << 31) + 1502),
            (D - 2503, D)]
    host = [[t[:, lo:hi].cpu().numpy().copy() for t in (dx, dv, dp)] for lo, hi in wins]
    hpl = [np.full(K, np.inf, F32) for _ in wins]
    dpl = gh.to_dev(np.full(K, np.inf, F32))
    losses = np.array([[0.9, 0.4], [0.7, 0.5], [0.2, 0.6]], F32)   # g = 1, 1, 0; 2, 1, 1 rows improve
    h = pso.pso_ps_create(K, D)
    try:
        for s in range(3):
            x_old = dx.clone()
            pso.pso_ps_sync(h, dx, dv, dp, dpl, gh.to_dev(losses[s]), dg, w, c1, c2, seed, s)
            g_dev, imp_dev = pso.pso_ps_last_selection(h, K)
            for (lo, hi), (hx, hv, hp), pl in zip(wins, host, hpl):
                hg = np.empty(hi - lo, F32)
                g, improved = oracle.sync(hx, hv, hp, pl, losses[s], hg, F32(w), F32(c1), F32(c2),
                                          seed, s, d0=lo)
                what = f"long rows step {s} columns [{lo},{hi})"
                assert g_dev == g and imp_dev == [bool(t) for t in improved], what
                gh.assert_bits_equal(dg[lo:hi].cpu().numpy(), hg, what + ": gbest")
                gh.assert_bits_equal(dp[:, lo:hi].cpu().numpy(), hp, what + ": pbest")
                gh.assert_close(dx[:, lo:hi].cpu().numpy(), hx, what + ": x")
                gh.assert_close(dv[:, lo:hi].cpu().numpy(), hv, what + ": v")
            assert torch.equal(dg.view(torch.int32), x_old[g_dev].view(torch.int32)), "gbest != x_g"
            for i in range(K):          # row by row: keeps the temporaries at one row
                assert torch.equal(dx[i], x_old[i] + dv[i]), f"row {i}: x' != x + v'"
                assert bool((dv[i] != 0).any())
            del x_old
            print(f"[case] long rows step {s} ok (g={g_dev}, improved={sum(imp_dev)})", flush=True)
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)
