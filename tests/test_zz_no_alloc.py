"""The allocation-free entry point (pso_ps_sync_static, selection scratch in a
fixed device array inside the library) against the handle-based pso_ps_sync:
identical bits on two calls in a row, the second on a smaller swarm."""
import numpy as np
import pytest
import torch

import paper_2009_03816_amd as pso
from paper_2009_03816_amd import workloads as wl

import gpu_harness as gh

pytestmark = pytest.mark.gpu
F32 = np.float32


def both_ways(sw, steps, seed):
    K, D, ld = sw.cfg.K, sw.cfg.D, sw.ld
    fresh = lambda: [gh.to_dev(a) for a in (sw.x, sw.v, sw.pbest, sw.pbest_loss, np.zeros(D, F32))]
    ref, got = fresh(), fresh()
    h = pso.pso_ps_create(K, D, ld)
    # the reference takes the stage in two launches; the static call makes the
    # library's own choice, which is one launch for the small swarm
    pso.pso_ps_set_single_launch(h, 0)
    try:
        for s in range(steps):
            loss = gh.to_dev(sw.losses[s])
            pso.pso_ps_sync(h, ref[0], ref[1], ref[2], ref[3], loss, ref[4], 0.7, 1.5, 1.5, seed, s)
            pso.pso_ps_sync_static(0, K, D, ld, got[0], got[1], got[2], got[3], loss, got[4],
                                   0.7, 1.5, 1.5, seed, s)
            torch.cuda.synchronize()
            for name, a, b in zip(("x", "v", "pbest", "pbest_loss", "gbest"), ref, got):
                assert torch.equal(a.view(torch.int32), b.view(torch.int32)), \
                    f"K={K} D={D} step {s}: {name} differs from pso_ps_sync"
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


def test_static_entry_point_matches_the_handle_based_one():
    print("[case] allocation-free entry point: K=70 D=50,003, then K=5 D=4,098 (ld 4,100)", flush=True)
    both_ways(wl.small_swarm(70, 50_003, seed=71, steps=3), 3, seed=71)     # two mask words
    both_ways(wl.small_swarm(5, 4_098, seed=72, ld=4_100, steps=3), 3, seed=72)   # smaller, right after


def test_static_entry_point_at_its_largest_swarm():
    K = pso.PSO_PS_STATIC_MAX_K
    print(f"[case] allocation-free entry point: K={K} (64 words of improved flags) D=302", flush=True)
    both_ways(wl.small_swarm(K, 302, seed=73, steps=2), 2, seed=73)


def test_static_entry_point_rejects_what_it_cannot_hold():
    print("[case] allocation-free entry point: limits", flush=True)
    t = torch.zeros(64, dtype=torch.float32, device=gh.dev())
    p = t.data_ptr()
    with pytest.raises(pso.PsoPsError) as e:
        pso.pso_ps_sync_static(0, pso.PSO_PS_STATIC_MAX_K + 1, 4, 4, p, p, p, p, p, p,
                               0.5, 1.0, 1.0, 0, 0)
    assert e.value.code == pso.PSO_PS_ELIMIT and "scratch" in str(e.value)
    for bad in [dict(K=0, D=4, ld=4), dict(K=2, D=0, ld=4), dict(K=2, D=8, ld=4), dict(device=64)]:
        kw = {**dict(device=0, K=2, D=4, ld=4), **bad}
        with pytest.raises(pso.PsoPsError) as e:
            pso.pso_ps_sync_static(kw["device"], kw["K"], kw["D"], kw["ld"], p, p + 64, p + 128, p + 192,
                                   p + 200, p + 224, 0.5, 1.0, 1.0, 0, 0)
        assert e.value.code == pso.PSO_PS_EINVAL, bad
    with pytest.raises(pso.PsoPsError) as e:
        pso.pso_ps_sync_static(0, 2, 4, 4, None, p, p, p, p, p, 0.5, 1.0, 1.0, 0, 0)
    assert e.value.code == pso.PSO_PS_EINVAL
    torch.cuda.synchronize()
    assert not t.any()
