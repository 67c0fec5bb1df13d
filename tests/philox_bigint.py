"""Philox4x32-10 in Python arbitrary-precision integers, written from the
round definition of Salmon, Moraes, Dror and Shaw (SC'11), independently of
the C++ oracle: products are taken as whole integers and split by divmod, the
round keys are formed in closed form (k + r*W mod 2^32) instead of by running
addition, and the inverse round is provided so that tests can check that the
generator is the bijection the construction promises."""
import math

MASK = (1 << 32) - 1
M0 = 0xD2511F53
M1 = 0xCD9E8D57


def weyl_constants():
    """Key increments from their definitions: floor(2^32 * golden ratio
    fraction) and floor(2^32 * (sqrt(3) - 1)), by integer square roots."""
    w0 = (math.isqrt(5 << 64) - (1 << 32)) >> 1          # 2^32 (sqrt5 - 1)/2
    w1 = math.isqrt(3 << 64) - (1 << 32)                 # 2^32 (sqrt3 - 1)
    return w0 & MASK, w1 & MASK


W0, W1 = weyl_constants()


def round_fwd(c, k):
    hi0, lo0 = divmod(M0 * c[0], 1 << 32)
    hi1, lo1 = divmod(M1 * c[2], 1 << 32)
    return (hi1 ^ c[1] ^ k[0], lo1, hi0 ^ c[3] ^ k[1], lo0)


def round_inv(c, k):
    # lo words are M*c mod 2^32 with M odd, hence invertible.
    c2 = (c[1] * pow(M1, -1, 1 << 32)) & MASK
    c0 = (c[3] * pow(M0, -1, 1 << 32)) & MASK
    hi1 = (M1 * c2) >> 32
    hi0 = (M0 * c0) >> 32
    return (c0, c[0] ^ hi1 ^ k[0], c2, c[2] ^ hi0 ^ k[1])


def round_key(key, r):
    return ((key[0] + r * W0) & MASK, (key[1] + r * W1) & MASK)


def philox4x32_10(ctr, key):
    c = tuple(int(t) & MASK for t in ctr)
    for r in range(10):
        c = round_fwd(c, round_key(key, r))
    return c


def philox4x32_10_inverse(out, key):
    c = tuple(int(t) & MASK for t in out)
    for r in reversed(range(10)):
        c = round_inv(c, round_key(key, r))
    return c


def draw_r_exact(seed, step, i, d):
    """(r1, r2) for particle i, flat coordinate d as exact Fractions."""
    from fractions import Fraction
    out = philox4x32_10(((d >> 1) & MASK, i, step & MASK, (step >> 32) & MASK),
                        (seed & MASK, (seed >> 32) & MASK))
    j = d & 1
    return Fraction(out[2 * j] >> 8, 1 << 24), Fraction(out[2 * j + 1] >> 8, 1 << 24)
