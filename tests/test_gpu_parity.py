"""GPU parity: the HIP library, called through its C ABI, against the CPU
oracle on the same seeded inputs.  Bar: identical g, improved flags,
pbest_loss, pbest and gbest; x and v within 1e-6 relative (and, by design,
identical in bits)."""
import numpy as np
import pytest
import torch

import paper_2009_03816_amd as pso
from paper_2009_03816_amd import workloads as wl

import gpu_harness as gh

pytestmark = pytest.mark.gpu
F32 = np.float32


def run_trajectory(oracle, sw, steps=None, **kw):
    pair = gh.Pair(sw, **kw)
    try:
        for s in range(sw.cfg.steps if steps is None else steps):
            g, improved = pair.step(oracle, s)
            pair.check(g, improved, f"{sw.cfg.name} step {s}")
    finally:
        pair.close()


@pytest.mark.parametrize("name", ["mlp", "lenet5", "resnet20"])
def test_config_trajectory(oracle, name, stage_launches):
    print(f"[case] config {name}, dense rows, {stage_launches}", flush=True)
    run_trajectory(oracle, wl.make_swarm(wl.CONFIGS[name]))


@pytest.mark.parametrize("name", ["mlp", "resnet20"])
def test_config_trajectory_padded_rows(oracle, name, stage_launches):
    cfg = wl.CONFIGS[name]
    ld = (cfg.D + 3) // 4 * 4 + 4
    print(f"[case] config {name}, ld={ld}, {stage_launches}", flush=True)
    run_trajectory(oracle, wl.make_swarm(cfg, ld=ld), steps=min(cfg.steps, 6))


def test_lenet5_segments_match_flat_and_oracle(oracle, stage_launches):
    """The ragged per-layer layout gives the bits of the flat layout."""
    cfg = wl.CONFIGS["lenet5"]
    print(f"[case] config lenet5, {len(cfg.segments)} segments", flush=True)
    sw = wl.make_swarm(cfg)
    sizes = list(cfg.segments)
    hx, hv, hp, hpl = sw.x.copy(), sw.v.copy(), sw.pbest.copy(), sw.pbest_loss.copy()
    hg = np.zeros(cfg.D, F32)
    dx, dv, dp = ([gh.to_dev(a) for a in wl.segment_views(t, sizes)] for t in (sw.x, sw.v, sw.pbest))
    dg = [torch.zeros(n, dtype=torch.float32, device=gh.dev()) for n in sizes]
    dpl = gh.to_dev(sw.pbest_loss)
    h = pso.pso_ps_create(cfg.K, cfg.D, cfg.D, seg_sizes=sizes)
    tables = [pso.pso_ps_pointer_table(t) for t in (dx, dv, dp, dg)]
    try:
        for s in range(cfg.steps):
            w, c1, c2 = float(sw.w[s]), float(sw.c1), float(sw.c2)
            # lists of tensors, or pointer tables marshalled once: the same call
            a = (dx, dv, dp, dg) if s % 2 == 0 else tables
            pso.pso_ps_sync_segments(h, a[0], a[1], a[2], dpl, gh.to_dev(sw.losses[s]), a[3],
                                     w, c1, c2, cfg.seed, s)
            g, improved = oracle.sync(hx, hv, hp, hpl, sw.losses[s], hg, F32(w), F32(c1), F32(c2),
                                      cfg.seed, s)
            gg, gi = pso.pso_ps_last_selection(h, cfg.K)
            assert gg == g and gi == [bool(t) for t in improved]
            cat = lambda parts: np.concatenate([t.cpu().numpy() for t in parts], axis=-1)
            gh.assert_bits_equal(cat(dp), hp, f"segments step {s}: pbest")
            gh.assert_bits_equal(cat(dg), hg, f"segments step {s}: gbest")
            gh.assert_close(cat(dx), hx, f"segments step {s}: x")
            gh.assert_close(cat(dv), hv, f"segments step {s}: v")
            gh.assert_bits_equal(dpl.cpu().numpy(), hpl, f"segments step {s}: pbest_loss")
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


@pytest.mark.parametrize("sizes", [
    [5, 0, 1, 1024, 3, 4097, 2, 7],
    # more segments than one launch carries, ResNet-like: many small tensors and a few large ones
    [64, 64, 1728, 64, 64] * 14 + [0, 36_864, 1, 73_728, 128, 128, 10],
])
def test_odd_and_empty_segments(oracle, sizes, stage_launches):
    """Segment sizes that are odd (a Philox pair straddles two segments),
    one, and zero; several launches' worth of segments."""
    K, D = 5, sum(sizes)
    print(f"[case] odd segments K={K} sizes={sizes}", flush=True)
    sw = wl.small_swarm(K, D, seed=21, steps=3)
    hx, hv, hp, hpl = sw.x.copy(), sw.v.copy(), sw.pbest.copy(), sw.pbest_loss.copy()
    hg = np.zeros(D, F32)
    dx, dv, dp = ([gh.to_dev(a) for a in wl.segment_views(t, sizes)] for t in (sw.x, sw.v, sw.pbest))
    dg = [torch.zeros(max(n, 1), dtype=torch.float32, device=gh.dev())[:n] for n in sizes]
    dpl = gh.to_dev(sw.pbest_loss)
    h = pso.pso_ps_create(K, D, D, seg_sizes=sizes)
    try:
        for s in range(3):
            pso.pso_ps_sync_segments(h, dx, dv, dp, dpl, gh.to_dev(sw.losses[s]), dg,
                                     0.7, 1.5, 1.5, 21, s)
            oracle.sync(hx, hv, hp, hpl, sw.losses[s], hg, F32(0.7), F32(1.5), F32(1.5), 21, s)
            cat = lambda parts: np.concatenate([t.cpu().numpy() for t in parts], axis=-1)
            gh.assert_bits_equal(cat(dp), hp, f"odd segments step {s}: pbest")
            gh.assert_bits_equal(cat(dg), hg, f"odd segments step {s}: gbest")
            gh.assert_close(cat(dx), hx, f"odd segments step {s}: x")
            gh.assert_close(cat(dv), hv, f"odd segments step {s}: v")
            gh.assert_bits_equal(dpl.cpu().numpy(), hpl, f"odd segments step {s}: pbest_loss")
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(h)


@pytest.mark.parametrize("K,D,ld,offset", [
    (1, 1, 1, 0), (1, 7, 7, 0), (2, 2, 2, 0), (3, 3, 4, 0), (2, 5, 5, 0),       # tiny, odd
    (4, 1026, 1026, 0),                      # D = 2 mod 4: every other row is 8-byte aligned only
    (4, 1026, 1028, 0),                      # padded to 16-byte rows
    (3, 4099, 4099, 0),                      # odd D and stride: element-wise path
    (6, 2048 + 1, 2050, 0),                  # odd D, even stride: ragged last column
    (6, 2048 + 3, 2052, 0),                  # three ragged columns
    (5, 3000, 3000, 1),                      # buffers 4-byte aligned only
    (5, 3000, 3000, 2),                      # buffers 8-byte aligned only
    (33, 1500, 1500, 0), (64, 260, 260, 0), (65, 260, 260, 0), (130, 132, 132, 0),   # K beyond a wave
    (7, 70_000, 70_000, 0),                  # several workgroups and a ragged last one
    (40, 100_003, 100_003, 1),               # single launch: three particles per wavefront, 391 tiles
    # x, v, pbest and gbest at different offsets from a 16-byte boundary: 128-bit accesses
    # aligned in x only; odd offsets of x flip the parity of the random-number pairs
    (5, 3000, 3000, (0, 1, 2, 3)), (5, 3000, 3000, (1, 0, 3, 2)), (4, 5001, 5001, (3, 3, 0, 1)),
    (6, 4098, 4099, (2, 1, 1, 0)),           # odd stride: the parity alternates from row to row
    (9, 70_003, 70_005, (1, 2, 3, 0)),       # the same over several tiles per row
])
@pytest.mark.parametrize("stage", ["best_first", "copy", "single_launch"])
def test_shapes_and_alignments(oracle, K, D, ld, offset, stage):
    """The three shapes of the stage: selection + move of the best particle, then
    the others; selection + gbest copy, then all K; everything in one launch."""
    print(f"[case] K={K} D={D} ld={ld} offset={offset} stage={stage}", flush=True)
    sw = wl.small_swarm(K, D, seed=100 + K + D, ld=ld, steps=3)
    sw.x[:, D:] = 7.0; sw.v[:, D:] = 7.0; sw.pbest[:, D:] = 7.0     # padding must stay untouched
    if stage == "single_launch" and K > pso.PSO_PS_SINGLE_LAUNCH_MAX_K:
        with pytest.raises(pso.PsoPsError) as err:
            gh.Pair(sw, offset=offset, single_launch=1)
        assert err.value.code == pso.PSO_PS_ELIMIT
        return
    run_trajectory(oracle, sw, steps=3, offset=offset, best_first=stage != "copy",
                   single_launch=1 if stage == "single_launch" else 0)


@pytest.mark.parametrize("block,sup,chunk,wgs,generic", [
    (64, 0, 0, 0, False), (128, 0, 0, 0, False), (512, 0, 0, 0, False), (1024, 0, 0, 0, False),
    (64, 0, 0, 0, True), (256, 0, 0, 0, True),
    (64, 2, 1, 0, False), (64, 4, 4, 0, False), (64, 8, 2, 0, False), (128, 16, 16, 0, False),
    (256, 1, 1, 0, False), (64, 32, 8, 0, True),                         # XCD-aware orders
    (128, 0, 0, 3, False), (64, 0, 0, 8, False), (1024, 8, 2, 4, False), (256, 0, 0, 100, True)])
@pytest.mark.parametrize("best_first", [True, False])
def test_launch_shape_does_not_change_bits(oracle, block, sup, chunk, wgs, generic, best_first):
    print(f"[case] block={block} super={sup} chunk={chunk} wgs_per_cu={wgs} generic={generic} "
          f"best_first={best_first}", flush=True)
    sw = wl.small_swarm(9, 70_002, seed=5, steps=2)
    run_trajectory(oracle, sw, steps=2, block_threads=block, super_tiles=sup, chunk_tiles=chunk,
                   wgs_per_cu=wgs, force_generic=generic, best_first=best_first)


@pytest.mark.parametrize("origin", [1, 2])
@pytest.mark.parametrize("block,sup,chunk,offset,ld", [
    (64, 0, 0, 0, 70_002), (64, 8, 2, (3, 1, 2, 0), 70_003), (128, 4, 4, 258, 70_002),
    (256, 16, 1, (32, 0, 0, 0), 70_006), (64, 2, 1, 1, 70_002), (1024, 2, 2, 0, 70_002)])
def test_chunk_origin_does_not_change_bits(oracle, origin, block, sup, chunk, offset, ld):
    """Runs of tiles that start at absolute addresses: rows begin in the middle
    of a run, some workgroups name no tile."""
    print(f"[case] chunk origin {origin} block={block} super={sup} chunk={chunk} offset={offset} "
          f"ld={ld}", flush=True)
    sw = wl.small_swarm(9, 70_002, seed=6, ld=ld, steps=2)
    run_trajectory(oracle, sw, steps=2, offset=offset, block_threads=block, super_tiles=sup,
                   chunk_tiles=chunk, chunk_origin=origin, best_first=False)


def test_ties_nan_and_inf_losses(oracle, stage_launches):
    K, D = 8, 5000
    print(f"[case] ties / NaN / inf losses K={K} D={D}", flush=True)
    sw = wl.small_swarm(K, D, seed=77, steps=1)
    nan, inf = np.nan, np.inf
    tables = [
        [1.0, 0.5, 0.5, 2.0, 0.5, 3.0, 4.0, 5.0],          # three-way tie for the minimum
        [nan, nan, 0.7, nan, 0.7, nan, nan, nan],          # NaN never wins
        [1.0, 0.5, 0.5, 2.0, 0.4, 0.7, 4.0, nan],          # equal to own pbest_loss: no improvement
        [nan] * 8, [inf] * 8, [inf, -inf, 1.0, -inf, nan, 0.0, -0.0, 2.0],
    ]
    pair = gh.Pair(sw)
    try:
        for s, row in enumerate(tables):
            g, improved = pair.step(oracle, s, loss=np.array(row, F32))
            pair.check(g, improved, f"loss table {s}")
    finally:
        pair.close()


def test_random_shapes_alignments_and_layouts(oracle, stage_launches):
    """Sixty seeded random cases: K, D, row stride, buffer offsets (which pick
    the 128-bit or the element-wise path and shift the tile phase), launch shape,
    and for every third case a ragged split of the columns."""
    rng = np.random.default_rng(2009_03816)
    for case in range(60):
        K = int(rng.choice([1, 2, 3, 5, 8, 17, 33, 70]))
        D = int(rng.integers(1, 6000))
        ld = D + int(rng.choice([0, 0, 1, 2, 3, 4, 30]))
        offset = int(rng.choice([0, 0, 1, 2, 3, 4, 32, 258]))
        block = int(rng.choice([0, 64, 128, 256, 1024]))
        sup = int(rng.choice([0, 0, 1, 2, 8]))
        chunk = int(rng.choice([0, 1, 2, 4])) if sup else 0
        seed = int(rng.integers(0, 2 ** 62))
        print(f"[case] random {case}: K={K} D={D} ld={ld} offset={offset} block={block} "
              f"super={sup} chunk={chunk}", flush=True)
        sw = wl.small_swarm(K, D, seed=1000 + case, ld=ld, steps=2)
        if case % 3 == 2 and D >= 4:
            cuts = np.sort(rng.choice(np.arange(1, D), size=min(D - 1, int(rng.integers(1, 6))),
                                      replace=False))
            sizes = [int(t) for t in np.diff(np.concatenate([[0], cuts, [D]]))]
            hx, hv, hp = sw.x[:, :D].copy(), sw.v[:, :D].copy(), sw.pbest[:, :D].copy()
            hpl, hg = sw.pbest_loss.copy(), np.zeros(D, F32)
            dx, dv, dp = ([gh.to_dev(a, offset) for a in wl.segment_views(t, sizes)]
                          for t in (hx, hv, hp))
            dg = [gh.to_dev(np.zeros(n, F32), offset) for n in sizes]
            dpl = gh.to_dev(hpl)
            h = pso.pso_ps_create(K, D, D, seg_sizes=sizes)
            try:
                pso.pso_ps_set_launch(h, block, sup, chunk, 0, False)
                for s in range(2):
                    pso.pso_ps_sync_segments(h, dx, dv, dp, dpl, gh.to_dev(sw.losses[s]), dg,
                                             0.7, 1.5, 1.5, seed, s)
                    oracle.sync(hx, hv, hp, hpl, sw.losses[s], hg, F32(0.7), F32(1.5), F32(1.5),
                                seed, s)
                cat = lambda parts: np.concatenate([t.cpu().numpy() for t in parts], axis=-1)
                gh.assert_bits_equal(cat(dp), hp, f"random {case}: pbest")
                gh.assert_bits_equal(cat(dg), hg, f"random {case}: gbest")
                gh.assert_close(cat(dx), hx, f"random {case}: x")
                gh.assert_close(cat(dv), hv, f"random {case}: v")
            finally:
                torch.cuda.synchronize()
                pso.pso_ps_destroy(h)
        else:
            single = stage_launches == "single_launch" and K <= pso.PSO_PS_SINGLE_LAUNCH_MAX_K
            pair = gh.Pair(sw, offset=offset, block_threads=block, super_tiles=sup, chunk_tiles=chunk,
                           single_launch=1 if single else 0)
            try:
                for s in range(2):
                    g, improved = pair.step(oracle, s, seed=seed)
                pair.check(g, improved, f"random {case}")
            finally:
                pair.close()


def test_seed_and_step_use_all_64_bits(oracle, stage_launches):
    print("[case] 64-bit seed and step", flush=True)
    K, D = 3, 4100
    sw = wl.small_swarm(K, D, seed=19, steps=1)
    results = []
    for seed, step in [((1 << 63) + 5, (1 << 40) + 3), (5, (1 << 40) + 3), ((1 << 63) + 5, 3), (5, 3)]:
        host = [sw.x.copy(), sw.v.copy(), sw.pbest.copy(), sw.pbest_loss.copy(), np.zeros(D, F32)]
        dev = [gh.to_dev(a) for a in host]
        h = pso.pso_ps_create(K, D)
        try:
            pso.pso_ps_sync(h, dev[0], dev[1], dev[2], dev[3], gh.to_dev(sw.losses[0]), dev[4],
                            0.7, 1.5, 1.5, seed, step)
            oracle.sync(host[0], host[1], host[2], host[3], sw.losses[0], host[4], F32(0.7), F32(1.5),
                        F32(1.5), seed, step)
            gh.assert_close(dev[0].cpu().numpy(), host[0], f"seed {seed} step {step}: x")
            gh.assert_close(dev[1].cpu().numpy(), host[1], f"seed {seed} step {step}: v")
            results.append(host[1].copy())
        finally:
            torch.cuda.synchronize()
            pso.pso_ps_destroy(h)
    for a in range(4):
        for b in range(a + 1, 4):
            assert not np.array_equal(results[a], results[b])   # the high halves matter


def test_subnormal_values_are_kept(oracle, stage_launches):
    """Positions and velocities in the subnormal range: both sides keep
    gradual underflow, so the bits still agree."""
    print("[case] subnormal inputs", flush=True)
    sw = wl.small_swarm(4, 6000, seed=8, steps=3, x_sigma=3e-39, v_sigma=1e-39)
    assert np.any((np.abs(sw.x) < 1.1754944e-38) & (sw.x != 0))
    run_trajectory(oracle, sw, steps=3)


def test_non_finite_positions_propagate(oracle, stage_launches):
    """inf and NaN in x, v: the same elements become NaN/inf on both sides
    (the bit pattern of a NaN is not part of the contract), the rest agrees in bits."""
    print("[case] non-finite positions", flush=True)
    K, D = 4, 5000
    sw = wl.small_swarm(K, D, seed=9, steps=2)
    sw.x[1, 7] = np.inf; sw.x[2, 100] = -np.inf; sw.v[3, 4000] = np.nan; sw.x[0, 4999] = np.nan
    sw.pbest[:] = sw.x
    pair = gh.Pair(sw)
    try:
        for s in range(2):
            pair.step(oracle, s)
            for dev_t, host in ((pair.dx, pair.hx), (pair.dv, pair.hv), (pair.dp, pair.hp),
                                (pair.dg, pair.hg)):
                got = dev_t.cpu().numpy()
                assert np.array_equal(np.isnan(got), np.isnan(host))
                ok = ~np.isnan(host)
                assert np.array_equal(gh.bits(got)[ok], gh.bits(host)[ok])
            assert np.isnan(pair.hx).sum() >= 2
    finally:
        pair.close()


def test_two_handles_on_two_streams(oracle, stage_launches):
    """Independent swarms on their own handles and streams do not disturb each other."""
    print("[case] two handles, two streams", flush=True)
    a, b = wl.small_swarm(5, 30_000, seed=13, steps=4), wl.small_swarm(7, 20_002, seed=14, steps=4)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(sa):
        pa = gh.Pair(a)
    with torch.cuda.stream(sb):
        pb = gh.Pair(b)
    try:
        res = []
        for s in range(4):
            with torch.cuda.stream(sa):
                ra = pa.step(oracle, s)
            with torch.cuda.stream(sb):
                rb = pb.step(oracle, s)
            res.append((ra, rb))
        torch.cuda.synchronize()
        pa.check(*res[-1][0], "handle A"); pb.check(*res[-1][1], "handle B")
    finally:
        pa.close(); pb.close()


def test_stage_can_be_captured_in_a_hip_graph(oracle, stage_launches):
    """A stage allocates nothing, copies nothing to the host and clears no
    memory, so it can be recorded into a HIP graph; every replay (with eager
    work and synchronisation in between) gives the bits of the eager call."""
    print("[case] HIP graph capture and replay", flush=True)
    K, D = 6, 50_002
    sw = wl.small_swarm(K, D, seed=17, steps=1)
    loss = gh.to_dev(sw.losses[0])

    def fresh():
        return [gh.to_dev(a) for a in (sw.x, sw.v, sw.pbest, sw.pbest_loss, np.zeros(D, F32))]

    def stage(h, st):
        pso.pso_ps_sync(h, st[0], st[1], st[2], st[3], loss, st[4], 0.7, 1.5, 1.5, 17, 3)

    eager, graphed = fresh(), fresh()
    he, hg = pso.pso_ps_create(K, D), pso.pso_ps_create(K, D)
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            stage(hg, graphed)                        # warm-up outside the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        for t, src in zip(graphed, fresh()):
            t.copy_(src)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            stage(hg, graphed)                        # recorded, not run
        for replay in range(3):
            stage(he, eager)
            graph.replay()
            torch.cuda.synchronize()
            scratch = torch.randn(1000, device=gh.dev()).sum().item()   # eager work in between
            assert scratch == scratch
            for te, tg in zip(eager, graphed):
                assert torch.equal(te.view(torch.int32), tg.view(torch.int32)), f"replay {replay}"
    finally:
        torch.cuda.synchronize()
        pso.pso_ps_destroy(he); pso.pso_ps_destroy(hg)


def test_deterministic_and_resumable(oracle, stage_launches):
    """Same (seed, step) gives the same bits; five stages, a new handle and
    five more equal ten stages in one go."""
    print("[case] determinism / resume", flush=True)
    cfg = wl.CONFIGS["mlp"]
    sw = wl.make_swarm(cfg, steps=10)

    def advance(state, h, lo, hi):
        for s in range(lo, hi):
            pso.pso_ps_sync(h, state[0], state[1], state[2], state[3], gh.to_dev(sw.losses[s]),
                            state[4], 0.7, 1.5, 1.5, 0, s)

    def fresh():
        return [gh.to_dev(a) for a in (sw.x, sw.v, sw.pbest, sw.pbest_loss, np.zeros(cfg.D, F32))]

    a, b = fresh(), fresh()
    ha = pso.pso_ps_create(cfg.K, cfg.D); advance(a, ha, 0, 10)
    hb = pso.pso_ps_create(cfg.K, cfg.D); advance(b, hb, 0, 5)
    torch.cuda.synchronize(); pso.pso_ps_destroy(hb)
    hb = pso.pso_ps_create(cfg.K, cfg.D); advance(b, hb, 5, 10)
    torch.cuda.synchronize()
    for ta, tb in zip(a, b):
        assert torch.equal(ta.view(torch.int32), tb.view(torch.int32))
    pso.pso_ps_destroy(ha); pso.pso_ps_destroy(hb)


@pytest.mark.parametrize("best_first,fused_rows,single", [(True, 0, 0), (False, 0, 0), (True, 2, 0),
                                                          (True, 0, 1), (False, 0, 1)])
def test_begin_then_finish_equals_sync(oracle, best_first, fused_rows, single):
    """pso_ps_sync_begin + pso_ps_sync_finish are the stage in two launches;
    pso_ps_sync is the same two launches (single = 0) or the whole stage in one."""
    print(f"[case] begin + finish == sync (best_first={best_first}, fused_rows={fused_rows}, "
          f"single_launch={single})", flush=True)
    sw = wl.small_swarm(6, 9000, seed=3, steps=1)
    one = [gh.to_dev(a) for a in (sw.x, sw.v, sw.pbest, sw.pbest_loss, np.zeros(9000, F32))]
    two = [gh.to_dev(a) for a in (sw.x, sw.v, sw.pbest, sw.pbest_loss, np.zeros(9000, F32))]
    loss = gh.to_dev(sw.losses[0])
    h = pso.pso_ps_create(6, 9000)
    pso.pso_ps_set_variant(h, fused_rows, 0, best_first)
    pso.pso_ps_set_single_launch(h, single)
    args = (0.7, 1.5, 1.5, 9, 4)
    pso.pso_ps_sync(h, one[0], one[1], one[2], one[3], loss, one[4], *args)
    pso.pso_ps_sync_begin(h, two[0], two[1], two[2], two[3], loss, two[4], *args)
    pso.pso_ps_sync_finish(h, two[0], two[1], two[2], two[3], loss, two[4], *args)
    torch.cuda.synchronize()
    for ta, tb in zip(one, two):
        assert torch.equal(ta.view(torch.int32), tb.view(torch.int32))
    pso.pso_ps_destroy(h)


def test_launch_shape_can_change_between_stages(oracle):
    """One launch, two launches, one again, ...: the ticket counters of the
    single launch are back at zero after every stage that used them."""
    print("[case] single launch and two launches alternating on one handle", flush=True)
    sw = wl.small_swarm(7, 12_345, seed=31, steps=6)
    pair = gh.Pair(sw)
    try:
        for s in range(6):
            pso.pso_ps_set_single_launch(pair.h, (1, 0, 1, 1, 0, -1)[s])
            g, improved = pair.step(oracle, s)
            pair.check(g, improved, f"alternating step {s}")
    finally:
        pair.close()


def test_runs_on_a_side_stream(oracle, stage_launches):
    print("[case] non-default stream", flush=True)
    sw = wl.small_swarm(4, 4096, seed=12, steps=1)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        run_trajectory(oracle, sw, steps=1)


def test_error_codes():
    print("[case] error codes", flush=True)
    with pytest.raises(pso.PsoPsError) as e:
        pso.pso_ps_create(0, 10)
    assert e.value.code == pso.PSO_PS_EINVAL
    for bad in [dict(K=2, D=0), dict(K=2, D=10, ld=9), dict(K=2, D=10, seg_sizes=[4, 5]),
                dict(K=2, D=10, seg_sizes=[11, -1])]:
        with pytest.raises(pso.PsoPsError) as e:
            pso.pso_ps_create(**bad)
        assert e.value.code == pso.PSO_PS_EINVAL, bad
    h = pso.pso_ps_create(2, 10)
    t = torch.zeros(1024, dtype=torch.float32, device=gh.dev())
    ok = t.data_ptr()
    args = lambda **kw: {**dict(x=ok, v=ok + 256, pbest=ok + 512, pbest_loss=ok + 768,
                                 loss=ok + 800, gbest=ok + 900), **kw}
    def call(**kw):
        a = args(**kw)
        pso.pso_ps_sync(h, a["x"], a["v"], a["pbest"], a["pbest_loss"], a["loss"], a["gbest"],
                        0.5, 1.0, 1.0, 0, 0)
    for name in ("x", "v", "pbest", "pbest_loss", "loss", "gbest"):
        with pytest.raises(pso.PsoPsError) as e:
            call(**{name: None})
        assert e.value.code == pso.PSO_PS_EINVAL, name
        with pytest.raises(pso.PsoPsError) as e:
            call(**{name: ok + 2})
        assert e.value.code == pso.PSO_PS_EALIGN, name
    with pytest.raises(pso.PsoPsError) as e:      # second half before any first half
        pso.pso_ps_sync_finish(h, ok, ok + 256, ok + 512, ok + 768, ok + 800, ok + 900,
                               0.5, 1.0, 1.0, 0, 0)
    assert e.value.code == pso.PSO_PS_EINVAL
    with pytest.raises(pso.PsoPsError) as e:      # flat handle has no segment table
        pso.pso_ps_sync_segments(h, [ok], [ok], [ok], ok, ok, [ok], 0.5, 1.0, 1.0, 0, 0)
    assert e.value.code == pso.PSO_PS_EINVAL
    for bad in [(100, 0, 0), (256, 3, 0), (256, 0, 6), (256, 0, 0, 2), (256, 0, 0, -1)]:
        with pytest.raises(pso.PsoPsError):
            pso.pso_ps_set_launch(h, *bad)
    for bad in (-2, 2):
        with pytest.raises(pso.PsoPsError) as e:
            pso.pso_ps_set_single_launch(h, bad)
        assert e.value.code == pso.PSO_PS_EINVAL
    big = pso.pso_ps_create(pso.PSO_PS_SINGLE_LAUNCH_MAX_K + 1, 10)
    with pytest.raises(pso.PsoPsError) as e:      # more particles than the single launch takes
        pso.pso_ps_set_single_launch(big, 1)
    assert e.value.code == pso.PSO_PS_ELIMIT
    pso.pso_ps_set_single_launch(big, -1)         # the default is always accepted
    pso.pso_ps_destroy(big)
    torch.cuda.synchronize()
    assert not t.any()                           # nothing was enqueued by the failed calls
    pso.pso_ps_destroy(h)
    pso.pso_ps_destroy(None)
