"""ctypes front end of the CPU oracle (``pso_ps_oracle.cpp``).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
CPU-baseline leg load this; the GPU library and its Python binding never do.
It marshals numpy arrays to the C++ oracle and adds no arithmetic of its own.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pso_ps_oracle.cpp")
_LIB = os.path.join(_HERE, "libpso_ps_oracle.so")

_CXXFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c++17", "-shared", "-fPIC",
             "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler; returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(["g++", *_CXXFLAGS, "-o", tmp, _SRC], check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u32p = ctypes.POINTER(ctypes.c_uint32)
        f32p = ctypes.POINTER(ctypes.c_float)
        lib.pso_ps_oracle_philox4x32_10.argtypes = [u32p, u32p, u32p]
        lib.pso_ps_oracle_philox4x32_10.restype = None
        lib.pso_ps_oracle_draw_r.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32,
                                             ctypes.c_uint64, f32p, f32p]
        lib.pso_ps_oracle_draw_r.restype = None
        lib.pso_ps_oracle_argmin.argtypes = [ctypes.c_int, f32p]
        lib.pso_ps_oracle_argmin.restype = ctypes.c_int
        lib.pso_ps_oracle_sync.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int64),
            ctypes.POINTER(ctypes.c_int64), ctypes.c_uint64,
            ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_void_p),
            ctypes.POINTER(ctypes.c_void_p), f32p, f32p, ctypes.POINTER(ctypes.c_void_p), f32p,
            ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_uint64, ctypes.c_uint64,
            ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_uint8),
            ctypes.POINTER(ctypes.c_int)]
        lib.pso_ps_oracle_sync.restype = ctypes.c_int
        lib.pso_ps_oracle_inertia.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_float,
                                              ctypes.c_float]
        lib.pso_ps_oracle_inertia.restype = ctypes.c_float
        lib.pso_ps_oracle_schedule.argtypes = [ctypes.c_int64] * 4 + [ctypes.c_float] * 4 + \
            [ctypes.POINTER(ctypes.c_int), f32p, f32p, f32p]
        lib.pso_ps_oracle_schedule.restype = ctypes.c_int
        lib.pso_ps_oracle_average.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int64, f32p,
                                              f32p]
        lib.pso_ps_oracle_average.restype = ctypes.c_int
        _lib = lib
    return _lib


def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> tuple:
    lib = _load()
    c = (ctypes.c_uint32 * 4)(*[int(t) & 0xFFFFFFFF for t in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(t) & 0xFFFFFFFF for t in key])
    o = (ctypes.c_uint32 * 4)()
    lib.pso_ps_oracle_philox4x32_10(c, k, o)
    return tuple(int(t) for t in o)


def draw_r(seed: int, step: int, i: int, d: int) -> tuple:
    """(r1, r2) of Eq. (6) as numpy float32 scalars."""
    lib = _load()
    r1, r2 = ctypes.c_float(), ctypes.c_float()
    lib.pso_ps_oracle_draw_r(seed, step, i, d, ctypes.byref(r1), ctypes.byref(r2))
    return np.float32(r1.value), np.float32(r2.value)


def argmin(loss: np.ndarray) -> int:
    lib = _load()
    loss = np.ascontiguousarray(loss, dtype=np.float32)
    return int(lib.pso_ps_oracle_argmin(loss.size,
                                        loss.ctypes.data_as(ctypes.POINTER(ctypes.c_float))))


def _check_rows(a: np.ndarray, K: int, n: int, name: str) -> int:
    if a.dtype != np.float32 or a.ndim != 2 or a.shape != (K, n):
        raise ValueError(f"{name}: need float32 [{K},{n}], got {a.dtype} {a.shape}")
    if a.strides[1] != 4 or a.strides[0] % 4 or not a.flags.writeable:
        raise ValueError(f"{name}: need unit column stride and a writable array")
    if K > 1 and a.strides[0] < 4 * n:
        raise ValueError(f"{name}: rows overlap")
    return a.strides[0] // 4 if K > 1 else max(n, 1)


def sync_segments(x_seg, v_seg, pbest_seg, pbest_loss: np.ndarray, loss: np.ndarray, gbest_seg,
                  w: float, c1: float, c2: float, seed: int, step: int, d0: int = 0,
                  gbest_loss: Optional[np.ndarray] = None):
    """One synchronization stage, in place, over lists of per-segment arrays.

    x_seg[s], v_seg[s], pbest_seg[s]: float32 [K, n_s] (rows may be strided);
    gbest_seg[s]: float32 [n_s]; pbest_loss, loss: float32 [K].
    gbest_loss: None for the best of this stage; a float32 [1] array (in/out)
    for the historical gBest, in which case gbest_seg is an input too.
    Returns (g, improved) with improved a uint8 [K] array, or
    (g, improved, replaced) when gbest_loss is given.
    """
    lib = _load()
    K = int(loss.shape[0])
    n_seg = len(x_seg)
    if not (len(v_seg) == len(pbest_seg) == len(gbest_seg) == n_seg):
        raise ValueError("segment lists differ in length")
    for a, name in ((pbest_loss, "pbest_loss"), (loss, "loss")):
        if a.dtype != np.float32 or a.shape != (K,) or not a.flags.c_contiguous:
            raise ValueError(f"{name}: need contiguous float32 [{K}]")
    sizes = (ctypes.c_int64 * n_seg)()
    lds = (ctypes.c_int64 * n_seg)()
    ptrs = [(ctypes.c_void_p * n_seg)() for _ in range(4)]
    for s in range(n_seg):
        n = int(x_seg[s].shape[1])
        ld = _check_rows(x_seg[s], K, n, f"x_seg[{s}]")
        for a, name in ((v_seg[s], "v_seg"), (pbest_seg[s], "pbest_seg")):
            if _check_rows(a, K, n, f"{name}[{s}]") != ld:
                raise ValueError(f"{name}[{s}]: row stride differs from x_seg[{s}]")
        gb = gbest_seg[s]
        if gb.dtype != np.float32 or gb.shape != (n,) or (n > 1 and gb.strides[0] != 4):
            raise ValueError(f"gbest_seg[{s}]: need contiguous float32 [{n}]")
        sizes[s], lds[s] = n, ld
        for arr, tab in zip((x_seg[s], v_seg[s], pbest_seg[s], gb), ptrs):
            tab[s] = arr.ctypes.data
    g = ctypes.c_int(-1)
    replaced = ctypes.c_int(-1)
    improved = np.zeros(K, dtype=np.uint8)
    f32p = ctypes.POINTER(ctypes.c_float)
    if gbest_loss is not None:
        if gbest_loss.dtype != np.float32 or gbest_loss.shape != (1,):
            raise ValueError("gbest_loss: need float32 [1]")
        gl = gbest_loss.ctypes.data_as(f32p)
    else:
        gl = None
    rc = lib.pso_ps_oracle_sync(
        K, n_seg, sizes, lds, d0, ptrs[0], ptrs[1], ptrs[2],
        pbest_loss.ctypes.data_as(f32p), loss.ctypes.data_as(f32p), ptrs[3], gl,
        w, c1, c2, seed, step, ctypes.byref(g),
        improved.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), ctypes.byref(replaced))
    if rc != 0:
        raise ValueError("pso_ps_oracle_sync rejected its arguments")
    if gbest_loss is not None:
        return int(g.value), improved, bool(replaced.value)
    return int(g.value), improved


def sync(x: np.ndarray, v: np.ndarray, pbest: np.ndarray, pbest_loss: np.ndarray,
         loss: np.ndarray, gbest: np.ndarray, w: float, c1: float, c2: float,
         seed: int, step: int, d0: int = 0, gbest_loss: Optional[np.ndarray] = None):
    """One synchronization stage, in place, on a flat swarm.

    x, v, pbest: float32 [K, n]; gbest: float32 [n]; the random numbers are
    those of flat coordinates d0 .. d0+n-1, so a column window of a larger
    swarm can be advanced on its own.  Returns (g, improved).
    """
    return sync_segments([x], [v], [pbest], pbest_loss, loss, [gbest], w, c1, c2, seed, step,
                         d0=d0, gbest_loss=gbest_loss)


def inertia(t: int, t_max: int, m_max: float, m_min: float) -> np.float32:
    """Eq. (5)."""
    return np.float32(_load().pso_ps_oracle_inertia(t, t_max, m_max, m_min))


def schedule(t: int, iteration_size: int, epoch_size: int, step: int, m_max: float, m_min: float,
             c1: float, c2: float):
    """(is_stage, w, c1/lambda, c2/lambda) of iteration t (1-based)."""
    flag = ctypes.c_int(-1)
    w, a1, a2 = ctypes.c_float(), ctypes.c_float(), ctypes.c_float()
    rc = _load().pso_ps_oracle_schedule(t, iteration_size, epoch_size, step, m_max, m_min, c1, c2,
                                        ctypes.byref(flag), ctypes.byref(w), ctypes.byref(a1),
                                        ctypes.byref(a2))
    if rc != 0:
        raise ValueError("pso_ps_oracle_schedule rejected its arguments")
    return bool(flag.value), np.float32(w.value), np.float32(a1.value), np.float32(a2.value)


def average(x: np.ndarray, mean: np.ndarray) -> None:
    """Parameter averaging in place: mean = column means of x, every row of x = mean."""
    K, n = x.shape
    ld = _check_rows(x, K, n, "x")
    if mean.dtype != np.float32 or mean.shape != (n,) or (n > 1 and mean.strides[0] != 4):
        raise ValueError(f"mean: need contiguous float32 [{n}]")
    f32p = ctypes.POINTER(ctypes.c_float)
    if _load().pso_ps_oracle_average(K, n, ld, x.ctypes.data_as(f32p), mean.ctypes.data_as(f32p)):
        raise ValueError("pso_ps_oracle_average rejected its arguments")
