"""Compiles csrc/pso_ps.hip into libpso_ps.so and csrc/stream_probes.hip into
libpso_ps_probes.so (both in-tree) with hipcc for gfx950."""
from __future__ import annotations

import hashlib
import os
import shutil
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
SOURCE = os.path.join(_PKG, "csrc", "pso_ps.hip")
INCLUDE = os.path.join(_ROOT, "include")
LIBRARY = os.path.join(_PKG, "libpso_ps.so")
PROBES_SOURCE = os.path.join(_PKG, "csrc", "stream_probes.hip")
PROBES_LIBRARY = os.path.join(_PKG, "libpso_ps_probes.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # the velocity update spells out its two fused multiply-adds; nothing else may fuse
    "-ffp-contract=off",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the HIP library cannot be built")
    return exe


def source_files() -> list:
    """Everything the stage's library is compiled from."""
    csrc = os.path.dirname(SOURCE)
    return [SOURCE, os.path.join(csrc, "tile_order.h"), os.path.join(INCLUDE, "pso_ps.h")]


def source_hash() -> str:
    """Hash of the bytes of the sources as they are on disk now.  The build
    stamps it into the library (pso_ps_source_hash), so that a library built
    from other sources can be told apart whatever the file times say."""
    digest = hashlib.sha256()
    for path in source_files():
        with open(path, "rb") as f:
            digest.update(os.path.basename(path).encode() + b"\0" + f.read() + b"\0")
    return digest.hexdigest()[:32]


def build_library(verbose: bool = False) -> str:
    """Always compiles; returns the path of the shared library."""
    tmp = LIBRARY + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), *HIPCC_FLAGS, f'-DPSO_PS_SOURCE_HASH="{source_hash()}"', "-I", INCLUDE,
           "-o", tmp, SOURCE]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIBRARY)
    return LIBRARY


def build_probes(verbose: bool = False) -> str:
    """Always compiles the stream probes (measurement only); returns the path."""
    tmp = PROBES_LIBRARY + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), *HIPCC_FLAGS, "-I", INCLUDE, "-o", tmp, PROBES_SOURCE]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    os.replace(tmp, PROBES_LIBRARY)
    return PROBES_LIBRARY


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_probes(verbose=True))
