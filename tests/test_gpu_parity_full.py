"""GPU parity at the full benchmark sizes, in the default launch shape.  The
oracle advances the WHOLE [K, D] state (its single-threaded routine on disjoint
column ranges from a thread pool, which is the single-threaded result bit for
bit) and every element of x, v, pbest and gbest is compared after every stage;
the selection rules and Eq. (7) are checked over the whole arrays as exact
properties as well."""
import gc

import numpy as np
import pytest
import torch

import paper_2009_03816_amd as pso
from paper_2009_03816_amd import workloads as wl

import gpu_harness as gh

pytestmark = pytest.mark.gpu
F32 = np.float32


def as_bits(t):
    return t.view(torch.int32)


@pytest.fixture(scope="module")
def large_swarm():
    """The K=32, D=25,557,032 swarm, drawn once for the tests below (which copy
    what they change)."""
    print("[case] drawing the resnet50x32 swarm", flush=True)
    sw = wl.make_swarm(wl.CONFIGS["resnet50x32"])
    yield sw
    del sw
    gc.collect()


def run_full_config(oracle, cfg, sw):
    K, D, name = cfg.K, cfg.D, cfg.name
    hx, hv, hp, hpl = sw.x.copy(), sw.v.copy(), sw.pbest.copy(), sw.pbest_loss.copy()
    hg = np.zeros(D, F32)
    dx, dv = gh.to_dev(sw.x), gh.to_dev(sw.v)
    dp = dx.clone()                                  # initial personal best = position (Algorithm 2)
    dpl = gh.to_dev(sw.pbest_loss)
    dg = torch.zeros(D, dtype=torch.float32, device=gh.dev())
    losses, w_tab, c1, c2 = sw.losses, sw.w, float(sw.c1), float(sw.c2)
    print("[case] swarm resident on the device", flush=True)
    h = pso.pso_ps_create(K, D)
    try:
        for s in range(cfg.steps):
            x_old, p_old = dx.clone(), dp.clone()
            w = float(w_tab[s])
            pso.pso_ps_sync(h, dx, dv, dp, dpl, gh.to_dev(losses[s]), dg, w, c1, c2, cfg.seed, s)
            g_dev, imp_dev = pso.pso_ps_last_selection(h, K)
            g, improved = gh.oracle_sync_whole(oracle, hx, hv, hp, hpl, losses[s], hg, w, c1, c2,
                                               cfg.seed, s)
            what = f"{name} step {s}"
            assert g_dev == g and imp_dev == [bool(t) for t in improved], what
            gh.assert_bits_equal(dpl.cpu().numpy(), hpl, what + ": pbest_loss")
            gh.assert_rows_match(dg, hg, what + ": gbest")
            gh.assert_rows_match(dp, hp, what + ": pbest")
            gh.assert_rows_match(dx, hx, what + ": x", close=True)
            gh.assert_rows_match(dv, hv, what + ": v", close=True)
            # whole arrays: Algorithm 3, Algorithm 1 and Eq. (7) as exact properties
            assert torch.equal(as_bits(dg), as_bits(x_old[g_dev])), "gbest != x_g before the move"
            for i in range(K):
                src = x_old[i] if imp_dev[i] else p_old[i]
                assert torch.equal(as_bits(dp[i]), as_bits(src)), f"pbest row {i}"
            assert torch.equal(dx, x_old + dv), "x' != x + v'"
            assert bool(torch.isfinite(dv).all())
            del x_old, p_old
            print(f"[case] {name} step {s} ok: every element (g={g_dev}, "
                  f"improved={sum(imp_dev)})", flush=True)
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


def test_full_size_vgg16(oracle):
    cfg = wl.CONFIGS["vgg16"]
    print(f"[case] full-size config vgg16: K={cfg.K} D={cfg.D}, all {cfg.steps} stages", flush=True)
    run_full_config(oracle, cfg, wl.make_swarm(cfg))


def test_full_size_resnet50x32(oracle, large_swarm):
    cfg = wl.CONFIGS["resnet50x32"]
    print(f"[case] full-size config resnet50x32: K={cfg.K} D={cfg.D}, all {cfg.steps} stages",
          flush=True)
    run_full_config(oracle, cfg, large_swarm)


def test_full_size_per_layer_layout(oracle, large_swarm):
    """The large swarm held as 161 per-tensor [K, n] arrays (six launches' worth
    of segments), two stages, every element against the oracle."""
    cfg = wl.CONFIGS["resnet50x32_layers"]
    K, D, sizes = cfg.K, cfg.D, list(cfg.segments)
    print(f"[case] full-size per-layer layout: K={K} D={D} in {len(sizes)} tensors", flush=True)
    sw = large_swarm
    hx, hv, hp, hpl = sw.x.copy(), sw.v.copy(), sw.pbest.copy(), sw.pbest_loss.copy()
    hg = np.zeros(D, F32)
    xs = [torch.from_numpy(a).to(gh.dev()) for a in wl.segment_views(sw.x, sizes)]
    vs = [torch.from_numpy(a).to(gh.dev()) for a in wl.segment_views(sw.v, sizes)]
    ps = [t.clone() for t in xs]
    gs = [torch.zeros(n, dtype=torch.float32, device=gh.dev()) for n in sizes]
    dpl = gh.to_dev(sw.pbest_loss)
    losses, c1, c2, w_tab = sw.losses, float(sw.c1), float(sw.c2), sw.w
    h = pso.pso_ps_create(K, D, D, seg_sizes=sizes)
    try:
        for step in range(2):
            x_old = [t.clone() for t in xs]
            w = float(w_tab[step])
            pso.pso_ps_sync_segments(h, xs, vs, ps, dpl, gh.to_dev(losses[step]), gs, w, c1, c2,
                                     cfg.seed, step)
            g_dev, imp_dev = pso.pso_ps_last_selection(h, K)
            g, improved = gh.oracle_sync_whole(oracle, hx, hv, hp, hpl, losses[step], hg, w, c1, c2,
                                               cfg.seed, step)
            what = f"per-layer step {step}"
            assert g_dev == g and imp_dev == [bool(t) for t in improved], what
            gh.assert_bits_equal(dpl.cpu().numpy(), hpl, what + ": pbest_loss")
            gh.assert_rows_match(torch.cat(gs), hg, what + ": gbest")
            gh.assert_rows_match(torch.cat(ps, dim=1), hp, what + ": pbest")
            gh.assert_rows_match(torch.cat(xs, dim=1), hx, what + ": x", close=True)
            gh.assert_rows_match(torch.cat(vs, dim=1), hv, what + ": v", close=True)
            for s in range(len(sizes)):
                assert torch.equal(as_bits(gs[s]), as_bits(x_old[s][g_dev]))
                assert torch.equal(xs[s], x_old[s] + vs[s]), f"tensor {s}: x' != x + v'"
            del x_old
            print(f"[case] per-layer step {step} ok: every element (g={g_dev}, "
                  f"improved={sum(imp_dev)})", flush=True)
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


def test_full_size_row_pointers(oracle, large_swarm):
    """K = 32 separately allocated rows of 25,557,032 columns, two stages, every element."""
    cfg = wl.CONFIGS["resnet50x32"]
    K, D = cfg.K, cfg.D
    print(f"[case] full-size row pointers: K={K} D={D}", flush=True)
    sw = large_swarm
    hx, hv, hp, hpl = sw.x.copy(), sw.v.copy(), sw.pbest.copy(), sw.pbest_loss.copy()
    hg = np.zeros(D, F32)
    xr = [torch.from_numpy(sw.x[i]).to(gh.dev()) for i in range(K)]
    vr = [torch.from_numpy(sw.v[i]).to(gh.dev()) for i in range(K)]
    pr = [t.clone() for t in xr]
    dpl, dg = gh.to_dev(sw.pbest_loss), torch.zeros(D, dtype=torch.float32, device=gh.dev())
    c1, c2, w = float(sw.c1), float(sw.c2), float(sw.w[0])
    h = pso.pso_ps_create(K, D)
    try:
        for step in range(2):
            pso.pso_ps_sync_rows(h, xr, vr, pr, dpl, gh.to_dev(sw.losses[step]), dg, w, c1, c2,
                                 cfg.seed, step)
            g_dev, imp_dev = pso.pso_ps_last_selection(h, K)
            g, improved = gh.oracle_sync_whole(oracle, hx, hv, hp, hpl, sw.losses[step], hg, w, c1,
                                               c2, cfg.seed, step)
            what = f"rows step {step}"
            assert g_dev == g and imp_dev == [bool(t) for t in improved], what
            gh.assert_bits_equal(dpl.cpu().numpy(), hpl, what + ": pbest_loss")
            gh.assert_rows_match(dg, hg, what + ": gbest")
            gh.assert_rows_match(pr, hp, what + ": pbest")
            gh.assert_rows_match(xr, hx, what + ": x", close=True)
            gh.assert_rows_match(vr, hv, what + ": v", close=True)
            print(f"[case] rows step {step} ok: every element", flush=True)
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


def test_full_size_history_and_averaging(oracle, large_swarm):
    """Historical gBest (three stages, the last of which keeps the old gbest) and
    parameter averaging of the positions they leave, every element."""
    cfg = wl.CONFIGS["resnet50x32"]
    K, D = cfg.K, cfg.D
    print(f"[case] full-size history + averaging: K={K} D={D}", flush=True)
    sw = large_swarm
    losses, c1, c2, w = sw.losses[:3].copy(), float(sw.c1), float(sw.c2), float(sw.w[0])
    losses[2] = losses[:2].min() + F32(1.0)          # a stage that keeps the old gbest
    hx, hv, hp, hpl = sw.x.copy(), sw.v.copy(), sw.pbest.copy(), sw.pbest_loss.copy()
    hg, hgl = np.zeros(D, F32), np.array([np.inf], F32)
    dx, dv = gh.to_dev(sw.x), gh.to_dev(sw.v)
    dp = dx.clone()
    dpl, dgl = gh.to_dev(sw.pbest_loss), gh.to_dev(np.array([np.inf], F32))
    dg = torch.zeros(D, dtype=torch.float32, device=gh.dev())
    h = pso.pso_ps_create(K, D)
    try:
        kept = 0
        for step in range(3):
            pso.pso_ps_sync_history(h, dx, dv, dp, dpl, gh.to_dev(losses[step]), dg, dgl, w, c1, c2,
                                    cfg.seed, step)
            g_dev, imp_dev, rep_dev = pso.pso_ps_last_selection(h, K, with_replaced=True)
            g, improved, rep = gh.oracle_sync_whole(oracle, hx, hv, hp, hpl, losses[step], hg, w, c1,
                                                    c2, cfg.seed, step, gbest_loss=hgl)
            what = f"history step {step}"
            assert (g_dev, imp_dev, rep_dev) == (g, [bool(t) for t in improved], rep), what
            gh.assert_bits_equal(dgl.cpu().numpy(), hgl, what + ": gbest_loss")
            gh.assert_bits_equal(dpl.cpu().numpy(), hpl, what + ": pbest_loss")
            gh.assert_rows_match(dg, hg, what + ": gbest")
            gh.assert_rows_match(dp, hp, what + ": pbest")
            gh.assert_rows_match(dx, hx, what + ": x", close=True)
            gh.assert_rows_match(dv, hv, what + ": v", close=True)
            kept += not rep_dev
            print(f"[case] history step {step} ok: every element (replaced={rep_dev})", flush=True)
        assert kept == 1

        dmean = torch.zeros(D, dtype=torch.float32, device=gh.dev())
        pso.pso_ps_average(h, dx, dmean)
        hmean = np.empty(D, F32)
        oracle.average(hx, hmean)
        gh.assert_rows_match(dmean, hmean, "mean")
        gh.assert_rows_match(dx, hx, "averaged rows")
        print("[case] averaging ok: every element", flush=True)
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


def test_rows_longer_than_2_to_31_columns(oracle):
    """Maximum sizes: two rows of 2^31 + 5,242,886 columns each (8.6 GB per row),
    so that column indices, byte offsets and the flat coordinate of the random
    numbers all pass 32 bits.  Inputs are drawn on the device (seeded); the
    oracle advances the whole state through the first stage (every element is
    compared) and, through all three stages, windows at the start, across column
    2^30 (byte offset 2^32), across column 2^31, and at the ragged end."""
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
    # the first stage is also compared on every one of the 4.3 G elements
    whole = [dx.cpu().numpy(), dv.cpu().numpy()]
    whole.append(whole[0].copy())
    whole_pl, whole_g = np.full(K, np.inf, F32), np.empty(D, F32)
    print("[case] long rows: whole state on the host", flush=True)
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
            if s == 0:
                g, improved = gh.oracle_sync_whole(oracle, whole[0], whole[1], whole[2], whole_pl,
                                                   losses[0], whole_g, w, c1, c2, seed, 0)
                assert g_dev == g and imp_dev == [bool(t) for t in improved]
                gh.assert_rows_match(dg, whole_g, "long rows, whole: gbest")
                gh.assert_rows_match(dp, whole[2], "long rows, whole: pbest")
                gh.assert_rows_match(dx, whole[0], "long rows, whole: x", close=True)
                gh.assert_rows_match(dv, whole[1], "long rows, whole: v", close=True)
                del whole, whole_g
                gc.collect()
                print("[case] long rows step 0 ok on every element", flush=True)
            assert torch.equal(dg.view(torch.int32), x_old[g_dev].view(torch.int32)), "gbest != x_g"
            for i in range(K):          # row by row: keeps the temporaries at one row
                assert torch.equal(dx[i], x_old[i] + dv[i]), f"row {i}: x' != x + v'"
                assert bool((dv[i] != 0).any())
            del x_old
            print(f"[case] long rows step {s} ok (g={g_dev}, improved={sum(imp_dev)})", flush=True)
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)
