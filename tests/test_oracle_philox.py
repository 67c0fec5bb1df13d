"""Pins of the oracle's random-number step: the generator itself, the counter
layout and the conversion to [0,1)."""
import ctypes
import os
import shutil
import subprocess
from fractions import Fraction

import numpy as np
import pytest

import philox_bigint as pb

HERE = os.path.dirname(os.path.abspath(__file__))


def test_weyl_constants_from_their_definition():
    # golden-ratio and sqrt(3)-1 fractions of 2^32, by integer square roots
    assert pb.W0 == 0x9E3779B9
    assert pb.W1 == 0xBB67AE85


def test_oracle_philox_matches_bigint_reference(oracle):
    rng = np.random.default_rng(1234)
    words = rng.integers(0, 1 << 32, size=(10000, 6), dtype=np.uint64)
    special = [(0,) * 6, (0xFFFFFFFF,) * 6, (1, 0, 0, 0, 0, 0), (0, 0, 0, 1, 0, 0),
               (0, 0, 0, 0, 1, 0), (0, 0, 0, 0, 0, 1)]
    for row in list(map(tuple, words)) + special:
        ctr, key = row[:4], row[4:]
        assert oracle.philox4x32_10(ctr, key) == pb.philox4x32_10(ctr, key)


def test_bigint_reference_is_a_bijection_with_working_inverse():
    # The construction is a keyed permutation of the 128-bit counter; a wrong
    # wiring of the round (swapped words, wrong xor partner) breaks the inverse.
    rng = np.random.default_rng(5)
    for row in rng.integers(0, 1 << 32, size=(300, 6), dtype=np.uint64):
        ctr, key = tuple(int(t) for t in row[:4]), tuple(int(t) for t in row[4:])
        assert pb.philox4x32_10_inverse(pb.philox4x32_10(ctr, key), key) == ctr


@pytest.fixture(scope="module")
def rocrand_host(tmp_path_factory):
    inc = "/opt/rocm/include/rocrand/rocrand_philox4x32_10.h"
    if shutil.which("g++") is None or not os.path.exists(inc):
        pytest.skip("rocRAND headers or g++ not available")
    so = str(tmp_path_factory.mktemp("rocrand") / "librocrand_philox_host.so")
    subprocess.run(["g++", "-O1", "-shared", "-fPIC", "-D__HIP_PLATFORM_AMD__",
                    "-I/opt/rocm/include", os.path.join(HERE, "rocrand_philox_host.cpp"),
                    "-o", so], check=True)
    lib = ctypes.CDLL(so)
    lib.rocrand_philox_next4.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64,
                                         ctypes.POINTER(ctypes.c_uint32)]
    lib.rocrand_philox_next4.restype = None
    return lib


def test_oracle_philox_matches_rocrand_engine(oracle, rocrand_host):
    """AMD's open-source rocRAND engine, run on the host: seed is the key, the
    subsequence is the high counter half, offset/4 the low counter half."""
    rng = np.random.default_rng(99)
    cases = [(0, 0, 0), (1, 0, 0), (0, 1, 0), (0, 0, 4), ((1 << 64) - 1, (1 << 64) - 1, 4 * 77)]
    for _ in range(2000):
        seed, sub = (int(t) for t in rng.integers(0, 1 << 64, size=2, dtype=np.uint64))
        ctr_lo = int(rng.integers(0, 1 << 62, dtype=np.uint64))
        cases.append((seed, sub, 4 * ctr_lo))
    out = (ctypes.c_uint32 * 4)()
    for seed, sub, off in cases:
        rocrand_host.rocrand_philox_next4(seed, sub, off, out)
        q = off // 4
        ctr = (q & pb.MASK, q >> 32, sub & pb.MASK, sub >> 32)
        key = (seed & pb.MASK, seed >> 32)
        assert tuple(out) == oracle.philox4x32_10(ctr, key), (seed, sub, off)


def test_draw_r_counter_layout_and_conversion(oracle):
    """r1, r2 of coordinate d: call p = d >> 1 with counter (p, i, step_lo,
    step_hi), key (seed_lo, seed_hi); words 2j, 2j+1 for j = d & 1; top 24
    bits scaled by 2^-24."""
    rng = np.random.default_rng(7)
    for _ in range(3000):
        seed, step = (int(t) for t in rng.integers(0, 1 << 64, size=2, dtype=np.uint64))
        i = int(rng.integers(0, 1 << 16))
        d = int(rng.integers(0, 1 << 33))
        r1, r2 = oracle.draw_r(seed, step, i, d)
        e1, e2 = pb.draw_r_exact(seed, step, i, d)
        assert Fraction(float(r1)) == e1 and Fraction(float(r2)) == e2
        assert 0.0 <= r1 < 1.0 and 0.0 <= r2 < 1.0
    # a pair of neighbouring coordinates shares one call: (2p, 2p+1) -> words 0..3
    out = pb.philox4x32_10((5, 3, 9, 0), (11, 0))
    got = oracle.draw_r(11, 9, 3, 10) + oracle.draw_r(11, 9, 3, 11)
    assert [Fraction(float(t)) for t in got] == [Fraction(o >> 8, 1 << 24) for o in out]


def test_draw_r_depends_on_every_key_field(oracle):
    base = oracle.draw_r(1, 2, 3, 4)
    assert oracle.draw_r(1, 2, 3, 4) == base
    for other in [(2, 2, 3, 4), (1, 3, 3, 4), (1, 2, 4, 4), (1, 2, 3, 5), (1, 2, 3, 6),
                  (1 + (1 << 32), 2, 3, 4), (1, 2 + (1 << 32), 3, 4)]:
        assert oracle.draw_r(*other) != base
