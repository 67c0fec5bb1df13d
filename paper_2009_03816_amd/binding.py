"""ctypes binding of libpso_ps.so: the functions of include/pso_ps.h under the
same names.  Argument marshalling only; every step of the synchronization
stage runs in the library's HIP kernels.  Array arguments are torch tensors on
the GPU (or anything with ``data_ptr()``) or raw device addresses as ints.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

from . import build as _build

PSO_PS_OK = 0
PSO_PS_EINVAL = -1
PSO_PS_EALIGN = -2
PSO_PS_EHIP = -3
PSO_PS_ENOMEM = -4
PSO_PS_ELIMIT = -5
PSO_PS_STATIC_MAX_K = 4096
PSO_PS_SINGLE_LAUNCH_MAX_K = 64
PSO_PS_SINGLE_LAUNCH_MAX_PARAMS = 1_000_000

_f32p = ctypes.c_void_p   # device addresses travel as plain pointers
_lib = None


class PsoPsError(RuntimeError):
    def __init__(self, code: int, where: str, hip_error: int = 0):
        self.code, self.hip_error = code, hip_error
        extra = f" (hipError {hip_error})" if hip_error else ""
        super().__init__(f"{where}: {pso_ps_strerror(code)} [{code}]{extra}")


def library_path() -> str:
    return _build.LIBRARY


def _built_from(path: str) -> Optional[str]:
    """The source hash stamped into the library file at `path`, read from the
    file's bytes (nothing is loaded or run); None if there is no stamp."""
    marker = b"pso_ps_source_hash="
    with open(path, "rb") as f:
        blob = f.read()
    at = blob.find(marker)
    if at < 0:
        return None
    return blob[at + len(marker):at + len(marker) + 32].decode("ascii", "replace")


def load():
    """Load the built library.  It is built first if it has never been built,
    and rebuilt if it was built from other sources than those on disk now
    (the build stamps a hash of the sources into it).  Raises if it can be
    neither found nor built: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIBRARY):
        _build.build_library()
    elif _built_from(_build.LIBRARY) != _build.source_hash():
        try:
            _build.build_library()
        except Exception as exc:
            raise RuntimeError(
                f"{_build.LIBRARY} was built from other sources than those in "
                f"{os.path.dirname(_build.SOURCE)} and could not be rebuilt: {exc}") from exc
    # torch first: the library then binds to the HIP runtime torch has already
    # loaded, so that torch's streams and allocations are valid in its calls.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_build.LIBRARY)
    lib.pso_ps_source_hash.argtypes = []
    lib.pso_ps_source_hash.restype = ctypes.c_char_p
    if lib.pso_ps_source_hash().decode() != _build.source_hash():
        raise RuntimeError(f"{_build.LIBRARY} does not match the sources it should be built from")
    P, I, I64, U64, F = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_uint64, ctypes.c_float
    PP = ctypes.POINTER(ctypes.c_void_p)
    lib.pso_ps_create.argtypes = [PP, I, I64, I64, I, ctypes.POINTER(I64), I]
    lib.pso_ps_sync.argtypes = [P, _f32p, _f32p, _f32p, _f32p, _f32p, _f32p, F, F, F, U64, U64, P]
    lib.pso_ps_sync_segments.argtypes = [P, PP, PP, PP, _f32p, _f32p, PP, F, F, F, U64, U64, P]
    lib.pso_ps_sync_begin.argtypes = lib.pso_ps_sync.argtypes
    lib.pso_ps_sync_finish.argtypes = lib.pso_ps_sync.argtypes
    lib.pso_ps_last_selection.argtypes = [P, ctypes.POINTER(I), ctypes.POINTER(U64), I,
                                          ctypes.POINTER(I)]
    lib.pso_ps_sync_history.argtypes = [P, _f32p, _f32p, _f32p, _f32p, _f32p, _f32p, _f32p,
                                        F, F, F, U64, U64, P]
    lib.pso_ps_sync_rows.argtypes = [P, PP, PP, PP, _f32p, _f32p, _f32p, F, F, F, U64, U64, P]
    lib.pso_ps_sync_segments_history.argtypes = [P, PP, PP, PP, _f32p, _f32p, PP, _f32p, F, F, F,
                                                 U64, U64, P]
    lib.pso_ps_sync_rows_history.argtypes = [P, PP, PP, PP, _f32p, _f32p, _f32p, _f32p, F, F, F,
                                             U64, U64, P]
    lib.pso_ps_sync_static.argtypes = [I, I, I64, I64, _f32p, _f32p, _f32p, _f32p, _f32p, _f32p,
                                       F, F, F, U64, U64, P]
    lib.pso_ps_average.argtypes = [P, _f32p, _f32p, P]
    lib.pso_ps_inertia.argtypes = [I64, I64, F, F]
    lib.pso_ps_inertia.restype = F
    lib.pso_ps_schedule.argtypes = [I64, I64, I64, I64, F, F, F, F, ctypes.POINTER(I),
                                    ctypes.POINTER(F), ctypes.POINTER(F), ctypes.POINTER(F)]
    lib.pso_ps_set_launch.argtypes = [P, I, I, I, I, I]
    lib.pso_ps_set_variant.argtypes = [P, I, I, I]
    lib.pso_ps_set_single_launch.argtypes = [P, I]
    lib.pso_ps_last_hip_error.argtypes = [P]
    lib.pso_ps_destroy.argtypes = [P]
    lib.pso_ps_strerror.argtypes = [I]
    for name in ("pso_ps_create", "pso_ps_sync", "pso_ps_sync_segments", "pso_ps_sync_begin",
                 "pso_ps_sync_finish", "pso_ps_last_selection", "pso_ps_set_launch", "pso_ps_set_variant",
                 "pso_ps_set_single_launch",
                 "pso_ps_sync_history", "pso_ps_sync_rows", "pso_ps_average", "pso_ps_schedule",
                 "pso_ps_sync_segments_history", "pso_ps_sync_rows_history", "pso_ps_sync_static",
                 "pso_ps_last_hip_error", "pso_ps_destroy"):
        getattr(lib, name).restype = I
    lib.pso_ps_strerror.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _addr(a) -> Optional[int]:
    if a is None:
        return None
    if isinstance(a, int):
        return a
    return int(a.data_ptr())


def _stream(stream) -> Optional[int]:
    """A torch stream, a raw hipStream_t as int, or None for torch's current stream."""
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def _table(ptrs: Sequence):
    if isinstance(ptrs, ctypes.Array):
        return ptrs
    return (ctypes.c_void_p * len(ptrs))(*[_addr(p) for p in ptrs])


def pso_ps_pointer_table(arrays: Sequence):
    """The host array of device pointers that the ragged and row-pointer calls
    take, built once from tensors (or raw addresses) whose memory stays where
    it is: passing it instead of the list saves the per-call marshalling.  The
    caller keeps the tensors alive."""
    return _table(list(arrays))


def _check(rc: int, where: str, h=None):
    if rc != PSO_PS_OK:
        raise PsoPsError(rc, where, pso_ps_last_hip_error(h) if h else 0)


def pso_ps_strerror(code: int) -> str:
    return load().pso_ps_strerror(code).decode()


def pso_ps_create(K: int, D: int, ld: Optional[int] = None, seg_sizes: Optional[Sequence[int]] = None,
                  device: int = 0) -> int:
    """Returns the handle (an opaque integer)."""
    lib = load()
    h = ctypes.c_void_p()
    n_seg = 0 if seg_sizes is None else len(seg_sizes)
    sizes = (ctypes.c_int64 * n_seg)(*seg_sizes) if n_seg else None
    rc = lib.pso_ps_create(ctypes.byref(h), K, D, D if ld is None else ld, n_seg, sizes, device)
    _check(rc, "pso_ps_create")
    return h.value


def pso_ps_sync(h: int, x, v, pbest, pbest_loss, loss, gbest, w: float, c1: float, c2: float,
                seed: int, step: int, stream=None) -> None:
    rc = load().pso_ps_sync(h, _addr(x), _addr(v), _addr(pbest), _addr(pbest_loss), _addr(loss),
                            _addr(gbest), w, c1, c2, seed, step, _stream(stream))
    _check(rc, "pso_ps_sync", h)


def pso_ps_sync_segments(h: int, x_seg, v_seg, pbest_seg, pbest_loss, loss, gbest_seg,
                         w: float, c1: float, c2: float, seed: int, step: int, stream=None) -> None:
    rc = load().pso_ps_sync_segments(h, _table(x_seg), _table(v_seg), _table(pbest_seg),
                                     _addr(pbest_loss), _addr(loss), _table(gbest_seg),
                                     w, c1, c2, seed, step, _stream(stream))
    _check(rc, "pso_ps_sync_segments", h)


def pso_ps_sync_begin(h: int, x, v, pbest, pbest_loss, loss, gbest, w: float, c1: float, c2: float,
                      seed: int, step: int, stream=None) -> None:
    rc = load().pso_ps_sync_begin(h, _addr(x), _addr(v), _addr(pbest), _addr(pbest_loss),
                                  _addr(loss), _addr(gbest), w, c1, c2, seed, step, _stream(stream))
    _check(rc, "pso_ps_sync_begin", h)


def pso_ps_sync_finish(h: int, x, v, pbest, pbest_loss, loss, gbest, w: float, c1: float, c2: float,
                       seed: int, step: int, stream=None) -> None:
    rc = load().pso_ps_sync_finish(h, _addr(x), _addr(v), _addr(pbest), _addr(pbest_loss),
                                   _addr(loss), _addr(gbest), w, c1, c2, seed, step, _stream(stream))
    _check(rc, "pso_ps_sync_finish", h)


def pso_ps_last_selection(h: int, K: int, with_replaced: bool = False):
    """(g, improved) with improved a list of K bools, plus whether gbest was
    rewritten if with_replaced.  Waits for the stream."""
    words = (K + 63) // 64
    g, replaced = ctypes.c_int(-1), ctypes.c_int(-1)
    mask = (ctypes.c_uint64 * words)()
    _check(load().pso_ps_last_selection(h, ctypes.byref(g), mask, words, ctypes.byref(replaced)),
           "pso_ps_last_selection", h)
    improved = [bool((mask[i >> 6] >> (i & 63)) & 1) for i in range(K)]
    if with_replaced:
        return int(g.value), improved, bool(replaced.value)
    return int(g.value), improved


def pso_ps_sync_history(h: int, x, v, pbest, pbest_loss, loss, gbest, gbest_loss, w: float, c1: float,
                        c2: float, seed: int, step: int, stream=None) -> None:
    rc = load().pso_ps_sync_history(h, _addr(x), _addr(v), _addr(pbest), _addr(pbest_loss),
                                    _addr(loss), _addr(gbest), _addr(gbest_loss), w, c1, c2,
                                    seed, step, _stream(stream))
    _check(rc, "pso_ps_sync_history", h)


def pso_ps_sync_rows(h: int, x_rows, v_rows, pbest_rows, pbest_loss, loss, gbest, w: float,
                     c1: float, c2: float, seed: int, step: int, stream=None) -> None:
    rc = load().pso_ps_sync_rows(h, _table(x_rows), _table(v_rows), _table(pbest_rows),
                                 _addr(pbest_loss), _addr(loss), _addr(gbest), w, c1, c2,
                                 seed, step, _stream(stream))
    _check(rc, "pso_ps_sync_rows", h)


def pso_ps_sync_segments_history(h: int, x_seg, v_seg, pbest_seg, pbest_loss, loss, gbest_seg,
                                 gbest_loss, w: float, c1: float, c2: float, seed: int, step: int,
                                 stream=None) -> None:
    rc = load().pso_ps_sync_segments_history(h, _table(x_seg), _table(v_seg), _table(pbest_seg),
                                             _addr(pbest_loss), _addr(loss), _table(gbest_seg),
                                             _addr(gbest_loss), w, c1, c2, seed, step,
                                             _stream(stream))
    _check(rc, "pso_ps_sync_segments_history", h)


def pso_ps_sync_rows_history(h: int, x_rows, v_rows, pbest_rows, pbest_loss, loss, gbest,
                             gbest_loss, w: float, c1: float, c2: float, seed: int, step: int,
                             stream=None) -> None:
    rc = load().pso_ps_sync_rows_history(h, _table(x_rows), _table(v_rows), _table(pbest_rows),
                                         _addr(pbest_loss), _addr(loss), _addr(gbest),
                                         _addr(gbest_loss), w, c1, c2, seed, step, _stream(stream))
    _check(rc, "pso_ps_sync_rows_history", h)


def pso_ps_sync_static(device: int, K: int, D: int, ld: int, x, v, pbest, pbest_loss, loss, gbest,
                       w: float, c1: float, c2: float, seed: int, step: int, stream=None) -> None:
    rc = load().pso_ps_sync_static(device, K, D, ld, _addr(x), _addr(v), _addr(pbest),
                                   _addr(pbest_loss), _addr(loss), _addr(gbest), w, c1, c2,
                                   seed, step, _stream(stream))
    _check(rc, "pso_ps_sync_static")


def pso_ps_average(h: int, x, mean, stream=None) -> None:
    _check(load().pso_ps_average(h, _addr(x), _addr(mean), _stream(stream)), "pso_ps_average", h)


def pso_ps_inertia(t: int, t_max: int, m_max: float, m_min: float) -> float:
    return float(load().pso_ps_inertia(t, t_max, m_max, m_min))


def pso_ps_schedule(t: int, iteration_size: int, epoch_size: int, step: int, m_max: float,
                    m_min: float, c1: float, c2: float):
    """(is_stage, w, c1/lambda, c2/lambda) of iteration t (1-based)."""
    flag = ctypes.c_int(-1)
    w, a1, a2 = ctypes.c_float(), ctypes.c_float(), ctypes.c_float()
    rc = load().pso_ps_schedule(t, iteration_size, epoch_size, step, m_max, m_min, c1, c2,
                                ctypes.byref(flag), ctypes.byref(w), ctypes.byref(a1),
                                ctypes.byref(a2))
    _check(rc, "pso_ps_schedule")
    return bool(flag.value), float(w.value), float(a1.value), float(a2.value)


def pso_ps_set_launch(h: int, block_threads: int = 0, super_tiles: int = 0, chunk_tiles: int = 0,
                      wgs_per_cu: int = 0, force_generic: bool = False) -> None:
    _check(load().pso_ps_set_launch(h, block_threads, super_tiles, chunk_tiles, wgs_per_cu,
                                    int(force_generic)), "pso_ps_set_launch", h)


def pso_ps_set_variant(h: int, fused_rows: int = 0, chunk_origin: int = 0,
                       best_first: bool = True) -> None:
    _check(load().pso_ps_set_variant(h, fused_rows, chunk_origin, int(best_first)),
           "pso_ps_set_variant", h)


def pso_ps_set_single_launch(h: int, mode: int = -1) -> None:
    _check(load().pso_ps_set_single_launch(h, mode), "pso_ps_set_single_launch", h)


def pso_ps_source_hash() -> str:
    """Hash of the sources the loaded library was built from."""
    return load().pso_ps_source_hash().decode()


def pso_ps_last_hip_error(h: int) -> int:
    return int(load().pso_ps_last_hip_error(h))


def pso_ps_destroy(h: Optional[int]) -> None:
    _check(load().pso_ps_destroy(h), "pso_ps_destroy")
