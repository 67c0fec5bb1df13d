"""ctypes binding of libpso_ps_probes.so (include/pso_ps_probes.h): the
arithmetic-free stream kernels the benchmark uses to print memory-system
ceilings.  Marshalling only; not part of the synchronization stage."""
from __future__ import annotations

import ctypes
import os

from . import build as _build

_lib = None


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(_build.PROBES_LIBRARY) or \
                os.path.getmtime(_build.PROBES_LIBRARY) < os.path.getmtime(_build.PROBES_SOURCE):
            _build.build_probes()
        import torch  # noqa: F401  (the HIP runtime torch loaded serves this library too)
        lib = ctypes.CDLL(_build.PROBES_LIBRARY)
        P, I, I64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        lib.pso_ps_probe_stream.argtypes = [I, P, P, P, P, I, I64, I64, I, I, I, I, I, I, I, I, I, I, P]
        lib.pso_ps_probe_stream.restype = I
        lib.pso_ps_probe_policy.argtypes = [P, P, P, P, I, I64, I64, I, I, I, I, I, P]
        lib.pso_ps_probe_policy.restype = I
        _lib = lib
    return _lib


MIXES = {"read": 0, "copy": 1, "inplace": 2}


def pso_ps_probe_stream(mix: str, x, v, pbest, sink, K: int, D: int, ld: int, block_threads: int = 128,
                        quads: int = 1, rows_per_wg: int = 1, chunked: bool = True,
                        super_tiles: int = 1024, chunk_tiles: int = 128, wgs_per_cu: int = 10,
                        nt_loads: bool = True, nt_stores: bool = True,
                        absolute_chunks: int = 0, stream: int = 0) -> None:
    rc = load().pso_ps_probe_stream(MIXES[mix], x.data_ptr(), v.data_ptr(), pbest.data_ptr(),
                                    sink.data_ptr(), K, D, ld, block_threads, quads, rows_per_wg,
                                    int(chunked), super_tiles, chunk_tiles, wgs_per_cu,
                                    int(nt_loads), int(nt_stores), int(absolute_chunks),
                                    stream or None)
    if rc != 0:
        raise RuntimeError(f"pso_ps_probe_stream: status {rc}")


POLICY_BITS = {"sc0": 1, "nt": 2, "sc1": 16}


def policy_bits(text: str) -> int:
    """'nt+sc1' -> 18; 'none' or '' -> 0."""
    return sum(POLICY_BITS[t] for t in text.split("+") if t and t != "none")


def pso_ps_probe_policy(x, v, pbest, sink, K: int, D: int, ld: int, super_tiles: int = 2048,
                        chunk_tiles: int = 256, wgs_per_cu: int = 20, load_policy: int = 2,
                        store_policy: int = 2, stream: int = 0) -> None:
    rc = load().pso_ps_probe_policy(x.data_ptr(), v.data_ptr(), pbest.data_ptr(), sink.data_ptr(),
                                    K, D, ld, super_tiles, chunk_tiles, wgs_per_cu, load_policy,
                                    store_policy, stream or None)
    if rc != 0:
        raise RuntimeError(f"pso_ps_probe_policy: status {rc}")
