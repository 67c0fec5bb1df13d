"""GPU parity of the companions of the stage: historical gBest, row-pointer
mode, parameter averaging, and a run driven by the paper's schedule
(Table II, Eq. (5), lambda, step = 10).  Same bar as the main parity tests."""
import numpy as np
import pytest
import torch

import paper_2009_03816_amd as pso
from paper_2009_03816_amd import workloads as wl

import gpu_harness as gh

pytestmark = pytest.mark.gpu
F32 = np.float32


def compare_state(dev, host, what):
    """dev / host: (x, v, pbest, pbest_loss, gbest) as device tensors / numpy arrays."""
    gh.assert_bits_equal(dev[3].cpu().numpy(), host[3], what + ": pbest_loss")
    gh.assert_bits_equal(dev[4].cpu().numpy(), host[4], what + ": gbest")
    gh.assert_bits_equal(dev[2].cpu().numpy(), host[2], what + ": pbest")
    gh.assert_close(dev[0].cpu().numpy(), host[0], what + ": x")
    gh.assert_close(dev[1].cpu().numpy(), host[1], what + ": v")


@pytest.mark.parametrize("K,D,steps", [(6, 10_242, 14), (8, 1_000_002, 6)])
def test_history_trajectory(oracle, K, D, steps, stage_launches):
    print(f"[case] historical gBest K={K} D={D}", flush=True)
    sw = wl.small_swarm(K, D, seed=31, steps=steps)
    losses = sw.losses.copy()
    losses[3] = losses[:3].min() + F32(0.5)          # a stage that cannot replace
    if steps > 8:
        losses[8] = 2.0; losses[8, 2] = losses[:8].min()   # ties the best so far: kept
        losses[9] = np.nan
    host = [sw.x.copy(), sw.v.copy(), sw.pbest.copy(), sw.pbest_loss.copy(), np.full(D, 3.0, F32)]
    hgl = np.array([np.inf], F32)
    dev = [gh.to_dev(a) for a in host]
    dgl = gh.to_dev(hgl)
    h = pso.pso_ps_create(K, D)
    kept = 0
    try:
        for s in range(steps):
            pso.pso_ps_sync_history(h, dev[0], dev[1], dev[2], dev[3], gh.to_dev(losses[s]), dev[4],
                                    dgl, 0.7, 1.2, 1.3, 31, s)
            g, improved, rep = oracle.sync(host[0], host[1], host[2], host[3], losses[s], host[4],
                                           F32(0.7), F32(1.2), F32(1.3), 31, s, gbest_loss=hgl)
            gg, gi, grep = pso.pso_ps_last_selection(h, K, with_replaced=True)
            what = f"history K={K} D={D} step {s}"
            assert (gg, gi, grep) == (g, [bool(t) for t in improved], rep), what
            gh.assert_bits_equal(dgl.cpu().numpy(), hgl, what + ": gbest_loss")
            compare_state(dev, host, what)
            kept += not rep
        assert 0 < kept < steps
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


@pytest.mark.parametrize("K,D,ld,offset,block,generic", [
    (1, 3, 3, 0, 0, False), (1, 5_000, 5_000, 0, 0, False), (2, 7, 7, 0, 0, False),
    (5, 4_098, 4_098, 0, 128, False), (7, 4_099, 4_099, 0, 0, False),
    (9, 70_002, 70_004, (1, 2, 3, 0), 0, False), (33, 1_500, 1_501, (2, 0, 1, 3), 256, False),
    (70, 300, 300, 0, 0, False), (6, 9_001, 9_001, 0, 0, True),
])
def test_best_first_variant(oracle, K, D, ld, offset, block, generic):
    """The stage split as (selection + move of the best particle, which writes
    gbest) + (move of the other K-1 particles) gives the oracle's bits, ties and
    NaN losses included."""
    print(f"[case] best first K={K} D={D} ld={ld} offset={offset} block={block} generic={generic}",
          flush=True)
    sw = wl.small_swarm(K, D, seed=400 + K, ld=ld, steps=5)
    sw.x[:, D:] = 7.0; sw.v[:, D:] = 7.0; sw.pbest[:, D:] = 7.0
    losses = sw.losses.copy()
    if K >= 5:
        losses[2, 3] = losses[2].min()               # a tie for the best
        losses[3, 1] = losses[:3, 1].min()           # equal to its own best so far: not improved
        losses[4] = np.nan
        losses[4, K - 1] = 0.001                     # the last particle is the best
    pair = gh.Pair(sw, offset=offset, block_threads=block, force_generic=generic, best_first=True)
    try:
        for s in range(5):
            g, improved = pair.step(oracle, s, loss=losses[s])
            pair.check(g, improved, f"best first step {s}")
    finally:
        pair.close()


@pytest.mark.parametrize("fused_rows,block", [(1, 0), (2, 64), (3, 128), (4, 256), (6, 0), (8, 64)])
@pytest.mark.parametrize("K,D,ld,offset", [
    (1, 3, 3, 0), (2, 7, 7, 0), (5, 4_098, 4_098, 0), (7, 4_099, 4_099, 0),      # K below / not a multiple of P
    (9, 70_002, 70_004, (1, 2, 3, 0)),         # odd start: three Philox calls per four columns
    (33, 1_500, 1_501, (2, 0, 1, 3)),          # odd stride
    (70, 300, 300, 0),                         # two words of improved flags
])
def test_single_pass_variant(oracle, fused_rows, block, K, D, ld, offset):
    """The single-pass kernels (one workgroup walks all K rows of its columns,
    gbest kept on chip) give the bits of the oracle as well, with history too."""
    print(f"[case] single pass P={fused_rows} block={block} K={K} D={D} ld={ld} offset={offset}",
          flush=True)
    sw = wl.small_swarm(K, D, seed=300 + K + fused_rows, ld=ld, steps=3)
    sw.x[:, D:] = 7.0; sw.v[:, D:] = 7.0; sw.pbest[:, D:] = 7.0
    pair = gh.Pair(sw, offset=offset, block_threads=block, fused_rows=fused_rows)
    try:
        for s in range(3):
            g, improved = pair.step(oracle, s)
            pair.check(g, improved, f"single pass step {s}")
    finally:
        pair.close()
    # historical gBest through the same kernels, with a stage that keeps the old gbest
    losses = sw.losses.copy()
    losses[1] = losses[0].min() + F32(0.5)
    host = [sw.x.copy(), sw.v.copy(), sw.pbest.copy(), sw.pbest_loss.copy(), np.full(D, 3.0, F32)]
    hgl = np.array([np.inf], F32)
    dev = [gh.to_dev(a) for a in host]
    dgl = gh.to_dev(hgl)
    h = pso.pso_ps_create(K, D, ld)
    try:
        pso.pso_ps_set_launch(h, block, 0, 0, 0, False)
        pso.pso_ps_set_variant(h, fused_rows, 0, True)
        reps = []
        for s in range(3):
            pso.pso_ps_sync_history(h, dev[0], dev[1], dev[2], dev[3], gh.to_dev(losses[s]), dev[4],
                                    dgl, 0.7, 1.2, 1.3, 31, s)
            g, improved, rep = oracle.sync(host[0][:, :D], host[1][:, :D], host[2][:, :D], host[3],
                                           losses[s], host[4], F32(0.7), F32(1.2), F32(1.3), 31, s,
                                           gbest_loss=hgl)
            gg, gi, grep = pso.pso_ps_last_selection(h, K, with_replaced=True)
            assert (gg, gi, grep) == (g, [bool(t) for t in improved], rep)
            gh.assert_bits_equal(dgl.cpu().numpy(), hgl, f"single pass history step {s}: gbest_loss")
            compare_state(dev, host, f"single pass history step {s}")
            reps.append(rep)
        assert reps[:2] == [True, False]
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


@pytest.mark.parametrize("K,D,offsets", [
    (5, 20_000, [0, 0, 0, 0, 0]),              # separately allocated rows, all vector path
    (5, 20_002, [0, 2, 0, 2, 2]),              # some rows 8-byte aligned only
    (4, 9_001, [0, 1, 0, 3]),                  # 4-byte aligned rows: odd parity of the random pairs
    (70, 3_000, [0] * 70),                     # two launches of row pointers (64 + 6)
    (33, 1_030, [2 * (i % 2) for i in range(33)]),
    (65, 1_030, [2 * (i % 2) for i in range(65)]),
])
def test_row_pointer_mode(oracle, K, D, offsets, stage_launches):
    print(f"[case] row pointers K={K} D={D} offsets={offsets[:6]}", flush=True)
    sw = wl.small_swarm(K, D, seed=41 + K, steps=3)
    if K >= 65:
        sw.losses[1, K - 1] = 0.01             # g in the second group of rows
    host = [sw.x.copy(), sw.v.copy(), sw.pbest.copy(), sw.pbest_loss.copy(), np.zeros(D, F32)]
    rows = [[gh.to_dev(a[i], offsets[i]) for i in range(K)] for a in (sw.x, sw.v, sw.pbest)]
    dpl, dg = gh.to_dev(sw.pbest_loss), gh.to_dev(np.zeros(D, F32))
    h = pso.pso_ps_create(K, D)
    try:
        for s in range(3):
            pso.pso_ps_sync_rows(h, rows[0], rows[1], rows[2], dpl, gh.to_dev(sw.losses[s]), dg,
                                 0.7, 1.5, 1.5, 7, s)
            g, improved = oracle.sync(host[0], host[1], host[2], host[3], sw.losses[s], host[4],
                                      F32(0.7), F32(1.5), F32(1.5), 7, s)
            gg, gi = pso.pso_ps_last_selection(h, K)
            assert (gg, gi) == (g, [bool(t) for t in improved])
            stack = lambda parts: torch.stack(parts)
            dev = [stack(rows[0]), stack(rows[1]), stack(rows[2]), dpl, dg]
            compare_state(dev, host, f"rows K={K} D={D} step {s}")
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


@pytest.mark.parametrize("K,D,offsets", [
    (5, 20_002, [0, 2, 1, 3, 0]),              # every alignment among the rows
    (70, 3_001, [i % 4 for i in range(70)]),   # two launches of row pointers, g moves between them
])
def test_row_pointer_mode_with_history(oracle, K, D, offsets, stage_launches):
    print(f"[case] row pointers + historical gBest K={K} D={D}", flush=True)
    steps = 6
    sw = wl.small_swarm(K, D, seed=43 + K, steps=steps)
    losses = sw.losses.copy()
    losses[1, K - 1] = 0.01                    # g in the last group of rows, a new best
    losses[2] = losses[:2].min() + F32(0.25)   # cannot replace
    losses[4, 0] = losses[:4].min()            # ties the best so far: kept
    host = [sw.x.copy(), sw.v.copy(), sw.pbest.copy(), sw.pbest_loss.copy(), np.full(D, 3.0, F32)]
    hgl = np.array([np.inf], F32)
    # v and pbest of a row sit at other alignments than its x
    rows = [[gh.to_dev(a[i], (offsets[i] + shift) % 4) for i in range(K)]
            for a, shift in ((sw.x, 0), (sw.v, 1), (sw.pbest, 2))]
    dpl, dg, dgl = gh.to_dev(sw.pbest_loss), gh.to_dev(host[4]), gh.to_dev(hgl)
    h = pso.pso_ps_create(K, D)
    kept = 0
    try:
        for s in range(steps):
            pso.pso_ps_sync_rows_history(h, rows[0], rows[1], rows[2], dpl, gh.to_dev(losses[s]), dg,
                                         dgl, 0.7, 1.5, 1.5, 7, s)
            g, improved, rep = oracle.sync(host[0], host[1], host[2], host[3], losses[s], host[4],
                                           F32(0.7), F32(1.5), F32(1.5), 7, s, gbest_loss=hgl)
            gg, gi, grep = pso.pso_ps_last_selection(h, K, with_replaced=True)
            what = f"rows+history K={K} D={D} step {s}"
            assert (gg, gi, grep) == (g, [bool(t) for t in improved], rep), what
            gh.assert_bits_equal(dgl.cpu().numpy(), hgl, what + ": gbest_loss")
            dev = [torch.stack(rows[0]), torch.stack(rows[1]), torch.stack(rows[2]), dpl, dg]
            compare_state(dev, host, what)
            kept += not rep
        assert kept >= 2
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


@pytest.mark.parametrize("sizes", [
    list(wl.LENET5_SEGMENTS),
    [64, 63, 1728, 1, 64] * 14 + [0, 36_864, 1, 73_729, 128, 127, 10],   # three launches, odd starts
])
def test_segments_with_history(oracle, sizes, stage_launches):
    K, D, steps = 6, sum(sizes), 6
    print(f"[case] segments + historical gBest K={K} D={D} in {len(sizes)} segments", flush=True)
    sw = wl.small_swarm(K, D, seed=47, steps=steps)
    losses = sw.losses.copy()
    losses[2] = losses[:2].min() + F32(0.25)   # cannot replace
    losses[4, 1] = losses[:4].min()            # ties the best so far: kept
    losses[5] = np.nan                         # nobody wins, nothing improves
    hx, hv, hp, hpl = sw.x.copy(), sw.v.copy(), sw.pbest.copy(), sw.pbest_loss.copy()
    hg, hgl = np.full(D, 3.0, F32), np.array([np.inf], F32)
    dx, dv, dp = ([gh.to_dev(a) for a in wl.segment_views(t, sizes)] for t in (sw.x, sw.v, sw.pbest))
    dg = [gh.to_dev(a) for a in wl.segment_views(hg, sizes)]
    dpl, dgl = gh.to_dev(sw.pbest_loss), gh.to_dev(hgl)
    h = pso.pso_ps_create(K, D, D, seg_sizes=sizes)
    kept = 0
    try:
        for s in range(steps):
            pso.pso_ps_sync_segments_history(h, dx, dv, dp, dpl, gh.to_dev(losses[s]), dg, dgl,
                                             0.6, 1.1, 1.4, 47, s)
            g, improved, rep = oracle.sync(hx, hv, hp, hpl, losses[s], hg, F32(0.6), F32(1.1),
                                           F32(1.4), 47, s, gbest_loss=hgl)
            gg, gi, grep = pso.pso_ps_last_selection(h, K, with_replaced=True)
            what = f"segments+history step {s}"
            assert (gg, gi, grep) == (g, [bool(t) for t in improved], rep), what
            gh.assert_bits_equal(dgl.cpu().numpy(), hgl, what + ": gbest_loss")
            cat = lambda parts: torch.cat(parts, dim=-1)
            compare_state([cat(dx), cat(dv), cat(dp), dpl, cat(dg)], [hx, hv, hp, hpl, hg], what)
            kept += not rep
        assert kept >= 3
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


@pytest.mark.parametrize("K,D,ld,offset", [(1, 5, 5, 0), (2, 1_000, 1_000, 0), (5, 4_099, 4_099, 0),
                                           (7, 70_001, 70_004, 1), (32, 33_333, 33_336, 0),
                                           (16, 272_474, 272_474, 2)])
def test_parameter_averaging(oracle, K, D, ld, offset):
    print(f"[case] averaging K={K} D={D} ld={ld} offset={offset}", flush=True)
    sw = wl.small_swarm(K, D, seed=51 + K, ld=ld, steps=1)
    sw.x[:, D:] = 7.0
    hx, hmean = sw.x.copy(), np.zeros(D, F32)
    dx, dmean = gh.to_dev(sw.x, offset), gh.to_dev(np.zeros(D, F32), offset)
    h = pso.pso_ps_create(K, D, ld)
    try:
        pso.pso_ps_average(h, dx, dmean)
        oracle.average(hx[:, :D], hmean)
        gh.assert_bits_equal(dmean.cpu().numpy(), hmean, "mean")
        gh.assert_bits_equal(dx.cpu().numpy(), hx, "rows after averaging")
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


def test_run_with_the_papers_schedule(oracle, stage_launches):
    """Table II constants, inertia by Eq. (5), lambda = epoch number, a stage
    every 10th iteration: the library's schedule drives the library, the
    oracle's schedule drives the oracle."""
    K, D = 16, 61_706
    it, ep, step = 234, 2, 10
    print(f"[case] paper schedule K={K} D={D}, {it * ep} iterations", flush=True)
    consts = (F32(0.9), F32(0.3), F32(0.2), F32(0.9))
    sw = wl.small_swarm(K, D, seed=61, steps=it * ep // step + 1, x_sigma=0.1, v_sigma=0.01)
    host = [sw.x.copy(), sw.v.copy(), sw.pbest.copy(), sw.pbest_loss.copy(), np.zeros(D, F32)]
    dev = [gh.to_dev(a) for a in host]
    h = pso.pso_ps_create(K, D)
    stages = 0
    try:
        for t in range(1, it * ep + 1):
            is_stage, w, a1, a2 = pso.pso_ps_schedule(t, it, ep, step, *consts)
            o_stage, ow, oa1, oa2 = oracle.schedule(t, it, ep, step, *consts)
            assert is_stage == o_stage
            if not is_stage:
                continue                       # (local training would run here)
            loss = sw.losses[stages]
            pso.pso_ps_sync(h, dev[0], dev[1], dev[2], dev[3], gh.to_dev(loss), dev[4],
                            w, a1, a2, 61, stages)
            oracle.sync(host[0], host[1], host[2], host[3], loss, host[4], ow, oa1, oa2, 61, stages)
            stages += 1
            if stages % 6 == 0 or stages < 3:
                compare_state(dev, host, f"paper schedule stage {stages} (t={t})")
        assert stages == (it * ep - 1) // step
        compare_state(dev, host, "paper schedule, final state")
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)
