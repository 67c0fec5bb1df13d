"""IEEE binary32 rounding (nearest, ties to even, gradual underflow) of exact
rationals, so that a test can work Eq. (6), (7) in exact arithmetic and round
where the arithmetic rounds, without using any floating-point unit."""
from fractions import Fraction

import numpy as np

_EMIN, _P = -126, 24
_MAX = Fraction((1 << 24) - 1, 1 << 23) * Fraction(2) ** 127


def rnd(q: Fraction) -> Fraction:
    if q == 0:
        return Fraction(0)
    sign = -1 if q < 0 else 1
    a = abs(q)
    # exponent e with 2^e <= a < 2^(e+1)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    elif Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, _EMIN)
    ulp = Fraction(2) ** (e - (_P - 1))
    n, rem = divmod(a, ulp)
    n = int(n)
    if rem * 2 > ulp or (rem * 2 == ulp and (n & 1)):
        n += 1
    r = n * ulp
    if r > _MAX:
        raise OverflowError("beyond binary32 range")
    return sign * r


def frac(a) -> Fraction:
    """Exact value of a numpy float32 / Python float."""
    return Fraction(float(a))


def sub(a, b): return rnd(a - b)
def add(a, b): return rnd(a + b)
def mul(a, b): return rnd(a * b)
def fma(a, b, c): return rnd(a * b + c)


def to_f32(q: Fraction) -> np.float32:
    f = np.float32(float(q))
    assert Fraction(float(f)) == q, "value is not a binary32"
    return f
