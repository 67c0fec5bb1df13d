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

    def __init__(self, sw, offset=0, block_threads: int = 0, super_tiles: int = 0,
                 chunk_tiles: int = 0, wgs_per_cu: int = 0, force_generic: bool = False,
                 fused_rows: int = 0, chunk_origin: int = 0, best_first: bool = True,
                 single_launch=None):
        """offset: elements by which every device array is shifted inside its
        allocation, or four of them for x, v, pbest and gbest.  The launch-shape
        and variant switches concern the stage in two launches: a caller that
        sets one of them gets that stage unless it says otherwise
        (single_launch: None = the handle's default, else the mode of
        pso_ps_set_single_launch)."""
        self.sw, self.K, self.D, self.ld = sw, sw.cfg.K, sw.cfg.D, sw.ld
        self.hx, self.hv, self.hp = sw.x.copy(), sw.v.copy(), sw.pbest.copy()
        self.hpl = sw.pbest_loss.copy()
        self.hg = np.zeros(self.D, F32)
        offs = (offset,) * 4 if isinstance(offset, int) else tuple(offset)
        self.dx, self.dv, self.dp = (to_dev(a, o) for a, o in zip((sw.x, sw.v, sw.pbest), offs))
        self.dpl = to_dev(sw.pbest_loss)
        self.dg = torch.zeros(self.D + offs[3], dtype=torch.float32, device=dev())[offs[3]:]
        self.h = pso.pso_ps_create(self.K, self.D, self.ld)
        try:
            if block_threads or super_tiles or chunk_tiles or wgs_per_cu or force_generic:
                pso.pso_ps_set_launch(self.h, block_threads, super_tiles, chunk_tiles, wgs_per_cu,
                                      force_generic)
            if fused_rows or chunk_origin or not best_first:
                pso.pso_ps_set_variant(self.h, fused_rows, chunk_origin, best_first)
            shaped = (block_threads or super_tiles or chunk_tiles or wgs_per_cu or force_generic
                      or fused_rows or chunk_origin or not best_first)
            if single_launch is None and shaped:
                single_launch = 0
            if single_launch is not None:
                pso.pso_ps_set_single_launch(self.h, single_launch)
        except Exception:
            pso.pso_ps_destroy(self.h)
            self.h = None
            raise

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


# ---------------------------------------------------------------------------
# Whole arrays at the full benchmark sizes
# ---------------------------------------------------------------------------
def host_threads() -> int:
    import os
    return max(1, min(16, len(os.sched_getaffinity(0))))


def oracle_sync_whole(oracle, x, v, pbest, pbest_loss, loss, gbest, w, c1, c2, seed, step,
                      gbest_loss=None, d0: int = 0):
    """One oracle stage over ALL columns of a large swarm: the oracle's own
    single-threaded routine, called on disjoint column ranges from a thread
    pool (ctypes releases the GIL).  The update of a column never looks at
    another column and the random numbers are indexed by the flat coordinate
    (d0 = first column of the range), so this is the single-threaded result
    bit for bit; each range gets its own copy of the per-particle scalars,
    which every range updates identically.  Returns what oracle.sync returns."""
    from concurrent.futures import ThreadPoolExecutor
    n = x.shape[1]
    threads = host_threads()
    bounds = [n * t // threads for t in range(threads + 1)]
    loss = np.ascontiguousarray(loss, dtype=F32)
    pls = [pbest_loss.copy() for _ in range(threads)]
    gls = [None if gbest_loss is None else gbest_loss.copy() for _ in range(threads)]

    def work(t):
        lo, hi = bounds[t], bounds[t + 1]
        if hi == lo:
            return None
        return oracle.sync(x[:, lo:hi], v[:, lo:hi], pbest[:, lo:hi], pls[t], loss, gbest[lo:hi],
                           F32(w), F32(c1), F32(c2), seed, step, d0=d0 + lo, gbest_loss=gls[t])

    with ThreadPoolExecutor(threads) as pool:
        results = [r for r in pool.map(work, range(threads)) if r is not None]
    first = results[0]
    for r in results[1:]:
        assert r[0] == first[0] and np.array_equal(r[1], first[1]) and r[2:] == first[2:]
    used = [t for t in range(threads) if bounds[t + 1] > bounds[t]]
    for t in used[1:]:
        assert np.array_equal(bits(pls[t]), bits(pls[used[0]]))
    pbest_loss[:] = pls[used[0]]
    if gbest_loss is not None:
        gbest_loss[:] = gls[used[0]]
    return first


def assert_rows_match(dev_rows, host: np.ndarray, what: str, close: bool = False):
    """Every element of a device array (a [K, n] tensor, a list of K row
    tensors, or a 1-D tensor) against the oracle's host array.  The host rows
    are uploaded one at a time and compared on the device; a row that differs
    is downloaded and reported element-wise.  close: also state the 1e-6
    relative bar of x and v explicitly (bit equality of finite values implies it)."""
    if isinstance(dev_rows, torch.Tensor) and dev_rows.dim() == 1:
        dev_rows, host = [dev_rows], host.reshape(1, -1)
    for i in range(host.shape[0]):
        d = dev_rows[i]
        ref = torch.from_numpy(np.ascontiguousarray(host[i])).to(d.device)
        same = torch.equal(d.view(torch.int32), ref.view(torch.int32))
        if close:
            lim = REL_TOL * torch.maximum(d.abs(), ref.abs())
            within = bool(((d - ref).abs() <= lim).all())        # false for any NaN
            if not within:
                assert_close(d.cpu().numpy(), host[i], f"{what} row {i}")
                raise AssertionError(f"{what} row {i}: beyond {REL_TOL} relative")
        if not same:
            assert_bits_equal(d.cpu().numpy(), host[i], f"{what} row {i}")
            raise AssertionError(f"{what} row {i}: bits differ")
        del ref
