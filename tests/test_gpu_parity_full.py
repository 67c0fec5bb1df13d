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
