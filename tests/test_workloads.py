"""The seeded input recipe: shapes, determinism, and the structure the
configurations promise (ragged sizes, injected ties, inertia ramp)."""
import numpy as np

from paper_2009_03816_amd import workloads as wl


def test_config_shapes():
    c = wl.CONFIGS
    assert (c["mlp"].K, c["mlp"].D) == (4, 101_770)
    assert (c["lenet5"].K, c["lenet5"].D) == (8, 61_706) and len(c["lenet5"].segments) == 10
    assert sum(c["lenet5"].segments) == c["lenet5"].D
    assert (c["resnet20"].K, c["resnet20"].D) == (16, 272_474)
    assert (c["vgg16"].K, c["vgg16"].D) == (8, 14_728_266)
    assert (c["resnet50x32"].K, c["resnet50x32"].D) == (32, 25_557_032)
    layers = c["resnet50x32_layers"]
    assert len(layers.segments) == 161 and sum(layers.segments) == layers.D == 25_557_032
    assert layers.segments[0] == 64 * 3 * 49 and layers.segments[-2:] == (2_048_000, 1000)


def test_seeded_and_initial_state():
    a = wl.make_swarm(wl.CONFIGS["mlp"]); b = wl.make_swarm(wl.CONFIGS["mlp"])
    for name in ("x", "v", "pbest", "pbest_loss", "losses", "w"):
        assert np.array_equal(getattr(a, name), getattr(b, name))
    assert a.x.dtype == np.float32 and a.x.shape == (4, 101_770)
    assert not a.v.any() and np.array_equal(a.pbest, a.x) and np.all(np.isinf(a.pbest_loss))
    assert abs(float(a.x.std()) - 0.05) < 1e-3
    assert a.losses.shape == (5, 4) and a.losses.min() >= 0.1 and a.losses.max() <= 2.5
    p = wl.make_swarm(wl.CONFIGS["mlp"], ld=101_772)
    assert np.array_equal(p.x[:, :101_770], a.x) and not p.x[:, 101_770:].any()


def test_inertia_ramp_and_ties():
    cfg = wl.CONFIGS["resnet20"]
    w = wl.inertia_table(cfg, cfg.steps)
    assert w.dtype == np.float32 and w[-1] == np.float32(0.4) and np.all(np.diff(w) < 0)
    assert abs(float(w[0]) - (0.9 - 0.5 / 50)) < 1e-7
    cfg = wl.CONFIGS["vgg16"]
    losses = wl.draw_losses(cfg, np.random.default_rng(cfg.seed), cfg.steps)
    tied = [s for s in range(cfg.steps) if np.sum(losses[s] == losses[s].min()) > 1]
    assert len(tied) == 1 and tied[0] > 0
    s = tied[0]
    run_min = losses[:s].min(axis=0)
    assert np.any((losses[s] == run_min) & (losses[s] != losses[s].min()))
