"""Seeded synthetic swarms: the inputs of a PSO-PS synchronization run.

This module only draws numbers.  It holds none of the method's arithmetic and
is imported by the tests and the benchmark, which hand the same arrays to the
GPU library and to the CPU oracle.

The paper's workloads are the weight vectors of n data-parallel workers
(n = 4 ... 16 in Section IV) and their mini-batch training losses; the shapes
below stand in for them: flattened parameter counts of common image
classifiers, Gaussian weights of initialisation-like scale, and losses in the
range of a 10-class cross-entropy.  Initial personal bests follow Algorithm 2
(every particle starts as a clone of its worker's weights): pbest = x and
pbest_loss = +inf.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

# LeNet-5 parameter tensors in registration order: conv1 w/b, conv2 w/b,
# fc1 w/b, fc2 w/b, fc3 w/b.
LENET5_SEGMENTS = (6 * 1 * 5 * 5, 6, 16 * 6 * 5 * 5, 16, 400 * 120, 120, 120 * 84, 84, 84 * 10, 10)


def resnet50_segments() -> Tuple[int, ...]:
    """Sizes of the 161 parameter tensors of a ResNet-50 classifier (1000
    classes) in registration order: 7x7 stem, four stages of 3/4/6/3 bottleneck
    blocks (1x1, 3x3, 1x1 convolutions, each followed by a batch-norm weight and
    bias; a 1x1 projection in the first block of a stage), and the final linear
    layer.  They sum to 25,557,032."""
    sizes = []

    def conv(cout, cin, k):
        sizes.append(cout * cin * k * k)

    def bn(c):
        sizes.extend([c, c])

    conv(64, 3, 7); bn(64)
    inplanes = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            conv(planes, inplanes, 1); bn(planes)
            conv(planes, planes, 3); bn(planes)
            conv(planes * 4, planes, 1); bn(planes * 4)
            if b == 0:
                conv(planes * 4, inplanes, 1); bn(planes * 4)
            inplanes = planes * 4
    sizes.extend([1000 * 2048, 1000])
    return tuple(sizes)


@dataclass(frozen=True)
class SwarmConfig:
    name: str
    K: int                       # particles = simulated workers
    D: int                       # parameters per particle
    x_sigma: float               # x ~ N(0, x_sigma)
    v_sigma: float               # v ~ N(0, v_sigma); 0 means v = 0
    loss: Tuple                  # ("uniform", lo, hi) | ("lognormal", mean, sigma)
    w: Tuple[float, float]       # inertia at the first and after the last step (linear)
    c1: float
    c2: float
    steps: int
    seed: int
    segments: Optional[Tuple[int, ...]] = None   # ragged per-layer sizes summing to D
    ties: bool = False           # inject equal losses on ceil(10 %) of the steps


CONFIGS = {
    "mlp": SwarmConfig("mlp", K=4, D=784 * 128 + 128 + 128 * 10 + 10, x_sigma=0.05, v_sigma=0.0,
                       loss=("uniform", 0.1, 2.5), w=(0.7, 0.7), c1=1.5, c2=1.5, steps=5, seed=0),
    "lenet5": SwarmConfig("lenet5", K=8, D=sum(LENET5_SEGMENTS), x_sigma=0.1, v_sigma=0.01,
                          loss=("uniform", 0.05, 2.3), w=(0.5, 0.5), c1=1.0, c2=2.0, steps=20,
                          seed=1, segments=LENET5_SEGMENTS),
    "resnet20": SwarmConfig("resnet20", K=16, D=272_474, x_sigma=0.05, v_sigma=0.005,
                            loss=("lognormal", 0.0, 0.5), w=(0.9, 0.4), c1=1.49, c2=1.49,
                            steps=50, seed=2),
    "vgg16": SwarmConfig("vgg16", K=8, D=14_728_266, x_sigma=0.02, v_sigma=0.0,
                         loss=("uniform", 0.2, 1.5), w=(0.7, 0.7), c1=1.5, c2=1.5, steps=10,
                         seed=3, ties=True),
    "resnet50x32": SwarmConfig("resnet50x32", K=32, D=25_557_032, x_sigma=0.02, v_sigma=0.002,
                               loss=("uniform", 0.5, 7.0), w=(0.72, 0.72), c1=1.49, c2=1.49,
                               steps=10, seed=4),
}
# The same swarm held as one dense [K, n] array per parameter tensor (161 of them).
CONFIGS["resnet50x32_layers"] = SwarmConfig(
    **{**CONFIGS["resnet50x32"].__dict__, "name": "resnet50x32_layers",
       "segments": resnet50_segments()})


@dataclass
class Swarm:
    cfg: SwarmConfig
    ld: int
    x: np.ndarray            # float32 [K, ld]; columns D..ld-1 are padding
    v: np.ndarray            # float32 [K, ld]
    pbest: np.ndarray        # float32 [K, ld]
    pbest_loss: np.ndarray   # float32 [K]
    losses: np.ndarray       # float32 [steps, K]
    w: np.ndarray            # float32 [steps]
    c1: np.float32 = field(default=np.float32(0))
    c2: np.float32 = field(default=np.float32(0))


def draw_losses(cfg: SwarmConfig, rng: np.random.Generator, steps: int) -> np.ndarray:
    kind = cfg.loss[0]
    if kind == "uniform":
        losses = rng.uniform(cfg.loss[1], cfg.loss[2], size=(steps, cfg.K))
    elif kind == "lognormal":
        losses = rng.lognormal(cfg.loss[1], cfg.loss[2], size=(steps, cfg.K))
    else:
        raise ValueError(kind)
    losses = losses.astype(np.float32)
    if cfg.ties and steps > 1 and cfg.K > 2:
        n_tie = -(-steps // 10)
        for s in rng.choice(np.arange(1, steps), size=min(n_tie, steps - 1), replace=False):
            # two particles share the minimum loss of this step ...
            lo = int(np.argmin(losses[s]))
            other = int(rng.choice([i for i in range(cfg.K) if i != lo]))
            losses[s, other] = losses[s, lo]
            # ... and a third one repeats the lowest loss it has had so far.
            third = int(rng.choice([i for i in range(cfg.K) if i not in (lo, other)]))
            losses[s, third] = losses[:s, third].min()
    return losses


def inertia_table(cfg: SwarmConfig, steps: int) -> np.ndarray:
    """Inertia handed to step s = 0..steps-1: a straight line from w[0] that
    reaches w[1] at the last of cfg.steps steps (constant when w[0] == w[1])."""
    s = np.arange(1, steps + 1, dtype=np.float64)
    return (cfg.w[0] - s * (cfg.w[0] - cfg.w[1]) / float(cfg.steps)).astype(np.float32) \
        if cfg.w[0] != cfg.w[1] else np.full(steps, cfg.w[0], dtype=np.float32)


def _normal_rows(rng: np.random.Generator, K: int, D: int, ld: int, sigma: float) -> np.ndarray:
    out = np.zeros((K, ld), dtype=np.float32)
    if sigma != 0.0:
        for i in range(K):
            row = rng.standard_normal(D, dtype=np.float32)
            row *= np.float32(sigma)
            out[i, :D] = row
    return out


def make_swarm(cfg: SwarmConfig, ld: Optional[int] = None, steps: Optional[int] = None) -> Swarm:
    """Draw the initial state and the per-step scalars of `cfg`.

    Draw order (fixed, so that a given seed always gives the same swarm):
    losses, x rows 0..K-1, v rows 0..K-1.
    """
    ld = cfg.D if ld is None else int(ld)
    if ld < cfg.D:
        raise ValueError("ld < D")
    steps = cfg.steps if steps is None else int(steps)
    rng = np.random.default_rng(cfg.seed)
    losses = draw_losses(cfg, rng, steps)
    x = _normal_rows(rng, cfg.K, cfg.D, ld, cfg.x_sigma)
    v = _normal_rows(rng, cfg.K, cfg.D, ld, cfg.v_sigma)
    return Swarm(cfg=cfg, ld=ld, x=x, v=v, pbest=x.copy(),
                 pbest_loss=np.full(cfg.K, np.inf, dtype=np.float32),
                 losses=losses, w=inertia_table(cfg, steps),
                 c1=np.float32(cfg.c1), c2=np.float32(cfg.c2))


def small_swarm(K: int, D: int, seed: int, ld: Optional[int] = None, steps: int = 3,
                x_sigma: float = 0.05, v_sigma: float = 0.01) -> Swarm:
    """A free-form swarm for edge-case tests (any K, D)."""
    cfg = SwarmConfig(f"small_{K}x{D}", K=K, D=D, x_sigma=x_sigma, v_sigma=v_sigma,
                      loss=("uniform", 0.1, 2.5), w=(0.7, 0.7), c1=1.5, c2=1.5, steps=steps,
                      seed=seed)
    return make_swarm(cfg, ld=ld)


def segment_views(a: np.ndarray, sizes) -> list:
    """Split the columns of a [K, >=sum(sizes)] (or [>=sum(sizes)]) array into
    dense per-segment copies, the layout of a per-layer parameter list."""
    out, start = [], 0
    for n in sizes:
        out.append(np.ascontiguousarray(a[..., start:start + n]))
        start += n
    return out
