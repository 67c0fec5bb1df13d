"""Shared plumbing of the GPU parity tests: put a seeded swarm on the device,
advance it with the library (through the C ABI binding) and with the CPU
oracle, and compare.  Holds no arithmetic of the method."""
from __future__ import annotations

import numpy as np
import torch

import paper_2009_03816_amd as pso

F32 = np.float32
REL_TOL = 1e-6     # the bar for x and v: |gpu - ref| <= REL_TOL * max(|gpu|, |ref|)


def dev():
    return torch.device("cuda:0")


def to_dev(a: np.ndarray, offset: int = 0) -> torch.Tensor:
    """Upload `a`; with offset > 0 the data starts that many elements into a
    larger allocation, which shifts its alignment."""
    flat = torch.empty(a.size + offset, dtype=torch.float32, device=dev())
    view = flat[offset:].view(a.shape)
    view.copy_(torch.from_numpy(np.ascontiguousarray(a)))
    return view


def bits(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a).view(np.uint32)


def assert_bits_equal(got: np.ndarray, want: np.ndarray, what: str):
    if not np.array_equal(bits(got), bits(want)):
        bad = np.argwhere(bits(got) != bits(want))
        first = tuple(bad[0])
        raise AssertionError(f"{what}: {len(bad)} of {got.size} elements differ in bits; first at "
                             f"{first}: gpu {got[first]!r} vs oracle {want[first]!r}")


def assert_close(got: np.ndarray, want: np.ndarray, what: str):
    """The stated bar for x and v (1e-6 relative) and, beyond it, the design
    goal of identical bits (same operation order, explicit fma on both sides)."""
    g64, w64 = got.astype(np.float64), want.astype(np.float64)
    err = np.abs(g64 - w64)
    lim = REL_TOL * np.maximum(np.abs(g64), np.abs(w64))
    if not np.all(err <= lim):
        i = tuple(np.argwhere(err > lim)[0])
        raise AssertionError(f"{what}: beyond {REL_TOL} relative at {i}: {got[i]!r} vs {want[i]!r}")
    assert_bits_equal(got, want, what)


class Pair:
    """One swarm held twice: on the device for the library, on the host for
    the oracle."""

    def __init__(self, sw, offset: int = 0, block_threads: int = 0, super_tiles: int = 0,
                 chunk_tiles: int = 0, wgs_per_cu: int = 0, force_generic: bool = False):
        self.sw, self.K, self.D, self.ld = sw, sw.cfg.K, sw.cfg.D, sw.ld
        self.hx, self.hv, self.hp = sw.x.copy(), sw.v.copy(), sw.pbest.copy()
        self.hpl = sw.pbest_loss.copy()
        self.hg = np.zeros(self.D, F32)
        self.dx, self.dv, self.dp = (to_dev(a, offset) for a in (sw.x, sw.v, sw.pbest))
        self.dpl = to_dev(sw.pbest_loss)
        self.dg = torch.zeros(self.D + offset, dtype=torch.float32, device=dev())[offset:]
        self.h = pso.pso_ps_create(self.K, self.D, self.ld)
        if block_threads or super_tiles or chunk_tiles or wgs_per_cu or force_generic:
            pso.pso_ps_set_launch(self.h, block_threads, super_tiles, chunk_tiles, wgs_per_cu,
                                  force_generic)

    def close(self):
        torch.cuda.synchronize()
        pso.pso_ps_destroy(self.h)
        self.h = None

    def step(self, oracle, s: int, seed=None, loss=None):
        sw = self.sw
        seed = sw.cfg.seed if seed is None else seed
        loss = sw.losses[s] if loss is None else loss
        w, c1, c2 = float(sw.w[min(s, len(sw.w) - 1)]), float(sw.c1), float(sw.c2)
        dloss = to_dev(loss)
        pso.pso_ps_sync(self.h, self.dx, self.dv, self.dp, self.dpl, dloss, self.dg,
                        w, c1, c2, seed, s)
        D = self.D
        g, improved = oracle.sync(self.hx[:, :D], self.hv[:, :D], self.hp[:, :D], self.hpl,
                                  np.ascontiguousarray(loss, dtype=F32), self.hg,
                                  F32(w), F32(c1), F32(c2), seed, s)
        return g, improved

    def check(self, g, improved, what: str):
        gg, gi = pso.pso_ps_last_selection(self.h, self.K)
        assert gg == g, f"{what}: g {gg} vs oracle {g}"
        assert gi == [bool(t) for t in improved], f"{what}: improved flags differ"
        assert_bits_equal(self.dpl.cpu().numpy(), self.hpl, f"{what}: pbest_loss")
        assert_bits_equal(self.dg.cpu().numpy(), self.hg, f"{what}: gbest")
        assert_bits_equal(self.dp.cpu().numpy(), self.hp, f"{what}: pbest")   # padding included
        assert_close(self.dx.cpu().numpy(), self.hx, f"{what}: x")
        assert_close(self.dv.cpu().numpy(), self.hv, f"{what}: v")
