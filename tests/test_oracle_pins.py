"""Pins of the oracle's synchronization stage against what the paper and the
mathematics fix: special cases of Eq. (6), (7), the selection rules of
Algorithms 1 and 3, exact-zero consequences, a float64 closed form with an
error bound, moments, and order independence."""
from fractions import Fraction

import numpy as np
import pytest

import exact_fp32 as ef
import philox_bigint as pb

F32 = np.float32


def rand_swarm(rng, K, D, ld=None, vscale=0.01):
    ld = D if ld is None else ld
    x = (rng.standard_normal((K, ld)) * 0.05).astype(F32)
    v = (rng.standard_normal((K, ld)) * vscale).astype(F32)
    pbest = (x + (rng.standard_normal((K, ld)) * 0.02).astype(F32)).astype(F32)
    pbest_loss = rng.uniform(0.5, 2.0, K).astype(F32)
    loss = rng.uniform(0.1, 2.5, K).astype(F32)
    gbest = np.full(D, np.nan, dtype=F32)
    return x, v, pbest, pbest_loss, loss, gbest


def run(oracle, x, v, pbest, pbest_loss, loss, gbest, w, c1, c2, seed, step, D=None, d0=0):
    D = gbest.shape[0] if D is None else D
    return oracle.sync(x[:, :D], v[:, :D], pbest[:, :D], pbest_loss, loss, gbest,
                       F32(w), F32(c1), F32(c2), seed, step, d0=d0)


def test_exact_rounder_agrees_with_ieee_conversion():
    """The rational rounder used below, checked against the hardware's
    float64 -> float32 conversion (one correctly rounded step)."""
    rng = np.random.default_rng(11)
    vals = np.concatenate([rng.standard_normal(2000), rng.standard_normal(500) * 1e-40,
                           [0.0, 1.0, 2.0 ** -149, 2.0 ** -150, 3 * 2.0 ** -150,
                            1 + 2.0 ** -24, 1 + 3 * 2.0 ** -24, 1 + 2.0 ** -24 + 2.0 ** -50]])
    for t in vals:
        assert ef.rnd(Fraction(float(t))) == Fraction(float(np.float32(t))), t


# -- Eq. (7) alone: w = 1, c1 = c2 = 0 gives v' = v, x' = x + v ---------------------------
def test_identity_case_is_x_plus_v(oracle):
    rng = np.random.default_rng(0)
    x, v, pbest, pl, loss, gb = rand_swarm(rng, 5, 37)
    x0, v0 = x.copy(), v.copy()
    run(oracle, x, v, pbest, pl, loss, gb, 1.0, 0.0, 0.0, 3, 4)
    assert np.array_equal(v.view(np.uint32), (v0 + F32(0)).view(np.uint32))
    assert np.array_equal(x.view(np.uint32), (x0 + v0).view(np.uint32))


# -- fixed point: all particles equal, pbest = x, v = 0 -> nothing moves ---------------------
def test_fixed_point(oracle):
    rng = np.random.default_rng(1)
    row = (rng.standard_normal(29) * 0.1).astype(F32)
    x = np.tile(row, (6, 1)); v = np.zeros_like(x); pbest = x.copy()
    pl = rng.uniform(0.1, 1, 6).astype(F32); loss = rng.uniform(0.1, 1, 6).astype(F32)
    gb = np.empty(29, F32)
    run(oracle, x, v, pbest, pl, loss, gb, 0.7, 1.5, 1.5, 8, 2)
    assert np.array_equal(x, np.tile(row, (6, 1))) and not v.any()
    assert np.array_equal(gb, row) and np.array_equal(pbest, x)


# -- Algorithm 3: gbest is the pre-move position of the first minimum-loss particle -----------
@pytest.mark.parametrize("K", [1, 2, 7, 33])
def test_gbest_is_first_argmin_row_before_move(oracle, K):
    rng = np.random.default_rng(K)
    x, v, pbest, pl, loss, gb = rand_swarm(rng, K, 19)
    if K > 2:
        loss[K - 1] = loss[1] = loss.min() / 2          # tie: lowest index wins
    x0 = x.copy()
    g, _ = run(oracle, x, v, pbest, pl, loss, gb, 0.7, 1.5, 1.5, 1, 1)
    assert g == int(np.argmin(loss)) == oracle.argmin(loss)
    assert np.array_equal(gb.view(np.uint32), x0[g].view(np.uint32))
    if K > 1:
        assert not np.array_equal(x[g], x0[g])          # the best particle moves too


def test_argmin_ignores_nan_and_defaults_to_zero(oracle):
    nan, inf = F32(np.nan), F32(np.inf)
    assert oracle.argmin(np.array([nan, 3, 1, nan, 1], F32)) == 2
    assert oracle.argmin(np.array([nan, nan, nan], F32)) == 0
    assert oracle.argmin(np.array([inf, inf], F32)) == 0
    assert oracle.argmin(np.array([inf, nan, -inf, -inf], F32)) == 2
    assert oracle.argmin(np.array([2, -0.0, 0.0], F32)) == 1


# -- Algorithm 1: strict "<" personal-best rule ----------------------------------------------
def test_pbest_rule(oracle):
    rng = np.random.default_rng(3)
    K, D = 6, 23
    x, v, pbest, pl, loss, gb = rand_swarm(rng, K, D)
    pl[:] = [1.0, 1.0, 1.0, np.inf, np.inf, 0.5]
    loss[:] = [0.5, 1.0, 1.5, np.inf, np.nan, 0.25]      # <, ==, >, inf vs inf, nan, <
    x0, p0, pl0 = x.copy(), pbest.copy(), pl.copy()
    g, improved = run(oracle, x, v, pbest, pl, loss, gb, 0.6, 1.0, 1.0, 2, 0)
    assert improved.tolist() == [1, 0, 0, 0, 0, 1]
    assert np.array_equal(pl, np.array([0.5, 1.0, 1.0, np.inf, np.inf, 0.25], F32))
    assert np.all(pl <= pl0)
    for i in range(K):
        want = x0[i] if improved[i] else p0[i]
        assert np.array_equal(pbest[i].view(np.uint32), want.view(np.uint32))
    assert g == 5


def test_pbest_loss_is_running_minimum_over_steps(oracle):
    rng = np.random.default_rng(4)
    K, D, steps = 5, 11, 12
    x, v, pbest, pl, _, gb = rand_swarm(rng, K, D)
    pl[:] = np.inf
    losses = rng.uniform(0.1, 2.5, (steps, K)).astype(F32)
    for s in range(steps):
        prev = pl.copy()
        run(oracle, x, v, pbest, pl, losses[s], gb, 0.7, 0.3, 0.3, 0, s)
        assert np.all(pl <= prev)
        assert np.array_equal(pl, losses[:s + 1].min(axis=0))


# -- exact zeros: best particle has no global term, improved particle no local term -------------
def test_exact_zero_terms(oracle):
    rng = np.random.default_rng(5)
    K, D = 4, 64
    x, v, pbest, pl, loss, gb = rand_swarm(rng, K, D)
    pl[:] = [1.0, 1.0, 1.0, 1.0]
    loss[:] = [2.0, 0.3, 0.9, 1.5]        # g = 1 (improved too), row 2 improved, rows 0, 3 not
    x0, v0, p0 = x.copy(), v.copy(), pbest.copy()
    w, c1, c2, seed, step = F32(0.7), F32(1.5), F32(1.25), 77, 5
    g, improved = run(oracle, x, v, pbest, pl, loss, gb, w, c1, c2, seed, step)
    assert g == 1 and improved.tolist() == [0, 1, 1, 0]
    r = np.array([[oracle.draw_r(seed, step, i, d) for d in range(D)] for i in range(K)], F32)
    # g and improved: v' = w v exactly (+0 added to a product keeps it, -0 aside)
    assert np.array_equal(v[1], w * v0[1] + F32(0))
    # improved only: v' = fma(a2, gbest - x, w v); evaluate the fma in float64 (exact
    # product of two binary32, one rounding from the sum is double rounding-safe here
    # only up to 1 ulp, so compare with the exact-rational rounding instead)
    for d in range(D):
        a2 = ef.mul(ef.frac(c2), ef.frac(r[2, d, 1]))
        dg = ef.sub(ef.frac(x0[1, d]), ef.frac(x0[2, d]))
        want = ef.fma(a2, dg, ef.mul(ef.frac(w), ef.frac(v0[2, d])))
        assert ef.frac(v[2, d]) == want
        # not improved, not g: all three terms
        a1 = ef.mul(ef.frac(c1), ef.frac(r[0, d, 0]))
        a2 = ef.mul(ef.frac(c2), ef.frac(r[0, d, 1]))
        dp = ef.sub(ef.frac(p0[0, d]), ef.frac(x0[0, d]))
        dg = ef.sub(ef.frac(x0[1, d]), ef.frac(x0[0, d]))
        acc = ef.fma(a1, dp, ef.mul(ef.frac(w), ef.frac(v0[0, d])))
        acc = ef.fma(a2, dg, acc)
        assert ef.frac(v[0, d]) == acc
        assert ef.frac(x[0, d]) == ef.add(ef.frac(x0[0, d]), acc)


# -- closed form of Eq. (6), (7) in float64 with the same r, error bound ------------------------
def test_float64_closed_form_bound(oracle):
    rng = np.random.default_rng(6)
    K, D = 7, 501
    x, v, pbest, pl, loss, gb = rand_swarm(rng, K, D)
    x0, v0, p0, pl0 = (a.astype(np.float64) for a in (x, v, pbest, pl))
    w, c1, c2, seed, step = F32(0.72), F32(1.49), F32(0.9), 2024, 31
    g, improved = run(oracle, x, v, pbest, pl, loss, gb, w, c1, c2, seed, step)
    r = np.array([[oracle.draw_r(seed, step, i, d) for d in range(D)] for i in range(K)],
                 np.float64)
    pb_new = np.where(improved[:, None].astype(bool), x0, p0)
    t0 = float(w) * v0
    t1 = float(c1) * r[..., 0] * (pb_new - x0)
    t2 = float(c2) * r[..., 1] * (x0[g][None, :] - x0)
    v_ref = t0 + t1 + t2
    x_ref = x0 + v_ref
    mag = np.abs(t0) + np.abs(t1) + np.abs(t2)
    eps = 2.0 ** -24
    assert np.all(np.abs(v.astype(np.float64) - v_ref) <= 3 * eps * mag + 1e-45)
    assert np.all(np.abs(x.astype(np.float64) - x_ref) <= 3 * eps * mag + eps * np.abs(x_ref) + 1e-45)


# -- signs: with v = 0, c1 = 0, c2 <= 1 every particle moves towards gbest, never past it ------
def test_moves_towards_gbest(oracle):
    rng = np.random.default_rng(7)
    K, D = 6, 400
    x, v, pbest, pl, loss, gb = rand_swarm(rng, K, D)
    v[:] = 0
    x0 = x.copy()
    g, _ = run(oracle, x, v, pbest, pl, loss, gb, 0.5, 0.0, 1.0, 5, 5)
    lo = np.minimum(x0, x0[g][None, :]); hi = np.maximum(x0, x0[g][None, :])
    assert np.all(x >= lo) and np.all(x <= hi)
    assert np.all(np.sign(x - x0) * np.sign(x0[g][None, :] - x0) >= 0)
    # and with c2 = 0, c1 <= 1, towards the personal best
    x, v, pbest, pl, loss, gb = rand_swarm(rng, K, D)
    v[:] = 0; pl[:] = 0.0                                 # nobody improves
    x0 = x.copy()
    run(oracle, x, v, pbest, pl, loss, gb, 0.5, 1.0, 0.0, 5, 5)
    lo = np.minimum(x0, pbest); hi = np.maximum(x0, pbest)
    assert np.all(x >= lo) and np.all(x <= hi) and np.any(x != x0)


# -- moments: x = 0, v = 0, gbest = 1, c1 = 0, c2 = 1  =>  x' = r2;  likewise r1 ---------------
def test_uniform_moments_through_the_stage(oracle):
    K, D = 4, 50000
    def draw(which, seed, step):
        x = np.zeros((K, D), F32); x[0] = 1.0            # row 0 will be g
        v = np.zeros((K, D), F32)
        pbest = np.ones((K, D), F32)
        pl = np.zeros(K, F32)                            # nobody improves
        loss = np.array([0.1, 1, 1, 1], F32)
        gb = np.empty(D, F32)
        c1, c2 = (1.0, 0.0) if which == 1 else (0.0, 1.0)
        run(oracle, x, v, pbest, pl, loss, gb, 0.0, c1, c2, seed, step)
        return x[1:].astype(np.float64)                  # rows 1..3: x' = r
    r1 = draw(1, 42, 0); r2 = draw(2, 42, 0); r2b = draw(2, 42, 1)
    n = r1.size
    for r in (r1, r2, r2b):
        assert r.min() >= 0.0 and r.max() < 1.0
        assert abs(r.mean() - 0.5) < 4 * np.sqrt(1 / 12 / n)
        assert abs(r.var() - 1 / 12) < 4 * np.sqrt(1 / 180 / n)
        ks = np.max(np.abs(np.sort(r.ravel()) - (np.arange(n) + 0.5) / n))
        assert ks < 1.95 / np.sqrt(n)
    def corr(a, b):
        return abs(np.corrcoef(a.ravel(), b.ravel())[0, 1])
    lim = 4 / np.sqrt(n)
    assert corr(r1, r2) < lim and corr(r2, r2b) < lim                 # r1 _|_ r2, step to step
    assert corr(r2[0], r2[1]) < 4 / np.sqrt(D)                        # particle to particle
    assert corr(r2[:, :-1], r2[:, 1:]) < lim                          # lag 1
    assert corr(r2[:, 0::2], r2[:, 1::2]) < 4 / np.sqrt(n / 2)        # within a call


# -- order independence / windows / strides / resume ----------------------------------------
def test_windows_strides_and_segments_agree(oracle):
    rng = np.random.default_rng(8)
    K, D = 5, 203
    x, v, pbest, pl, loss, gb = rand_swarm(rng, K, D)
    args = (F32(0.7), F32(1.5), F32(1.5), 9, 3)
    ref = [a.copy() for a in (x, v, pbest, pl, gb)]
    g_ref, imp_ref = oracle.sync(ref[0], ref[1], ref[2], ref[3], loss, ref[4], *args)
    # (a) padded rows
    ld = D + 5
    pad = [np.zeros((K, ld), F32) for _ in range(3)]
    for p, a in zip(pad, (x, v, pbest)):
        p[:, :D] = a
    pl2, gb2 = pl.copy(), gb.copy()
    oracle.sync(pad[0][:, :D], pad[1][:, :D], pad[2][:, :D], pl2, loss, gb2, *args)
    for p, r in zip(pad, ref[:3]):
        assert np.array_equal(p[:, :D].view(np.uint32), r.view(np.uint32)) and not p[:, D:].any()
    assert np.array_equal(pl2, ref[3]) and np.array_equal(gb2, ref[4])
    # (b) column windows advanced separately (odd and even starts)
    for lo, hi in [(0, 50), (50, 51), (51, 128), (128, 203)]:
        xs, vs, ps = (np.ascontiguousarray(a[:, lo:hi]) for a in (x, v, pbest))
        pl3, gb3 = pl.copy(), np.empty(hi - lo, F32)
        oracle.sync(xs, vs, ps, pl3, loss, gb3, *args, d0=lo)
        for got, r in zip((xs, vs, ps), ref[:3]):
            assert np.array_equal(got.view(np.uint32), r[:, lo:hi].view(np.uint32))
        assert np.array_equal(gb3, ref[4][lo:hi])
    # (c) ragged segments, including an odd-sized and an empty one
    sizes = [7, 0, 64, 1, 131]
    segs = [[np.ascontiguousarray(a[:, s:s + n]) for s, n in zip(np.cumsum([0] + sizes), sizes)]
            for a in (x, v, pbest)]
    gseg = [np.empty(n, F32) for n in sizes]
    pl4 = pl.copy()
    g4, imp4 = oracle.sync_segments(segs[0], segs[1], segs[2], pl4, loss, gseg, *args)
    assert g4 == g_ref and np.array_equal(imp4, imp_ref) and np.array_equal(pl4, ref[3])
    for got, r in zip(segs, ref[:3]):
        assert np.array_equal(np.concatenate(got, axis=1).view(np.uint32), r.view(np.uint32))
    assert np.array_equal(np.concatenate(gseg), ref[4])


def test_d_outer_brute_force_agrees(oracle):
    """The same stage with the loops the other way round (coordinate outer,
    particle inner), each coordinate advanced as its own window."""
    rng = np.random.default_rng(9)
    K, D = 4, 40
    x, v, pbest, pl, loss, gb = rand_swarm(rng, K, D)
    args = (F32(0.9), F32(0.2), F32(0.9), 1, 10)
    ref = [a.copy() for a in (x, v, pbest, pl, gb)]
    oracle.sync(ref[0], ref[1], ref[2], ref[3], loss, ref[4], *args)
    for d in range(D):
        cols = [np.ascontiguousarray(a[:, d:d + 1]) for a in (x, v, pbest)]
        g1 = np.empty(1, F32)
        oracle.sync(cols[0], cols[1], cols[2], pl.copy(), loss, g1, *args, d0=d)
        for got, r in zip(cols, ref[:3]):
            assert np.array_equal(got[:, 0].view(np.uint32), r[:, d].view(np.uint32))
        assert g1[0] == ref[4][d]


def test_same_seed_same_bits_and_resume(oracle):
    rng = np.random.default_rng(10)
    K, D, steps = 3, 50, 6
    x, v, pbest, pl, _, gb = rand_swarm(rng, K, D)
    pl[:] = np.inf
    losses = rng.uniform(0.1, 2.5, (steps, K)).astype(F32)
    def advance(state, lo, hi, seed=5):
        for s in range(lo, hi):
            oracle.sync(state[0], state[1], state[2], state[3], losses[s], state[4],
                        F32(0.7), F32(1.5), F32(1.5), seed, s)
    a = [t.copy() for t in (x, v, pbest, pl, gb)]; advance(a, 0, steps)
    b = [t.copy() for t in (x, v, pbest, pl, gb)]; advance(b, 0, 3)
    b = [t.copy() for t in b]; advance(b, 3, steps)
    c = [t.copy() for t in (x, v, pbest, pl, gb)]; advance(c, 0, steps, seed=6)
    for ta, tb in zip(a, b):
        assert np.array_equal(ta.view(np.uint32), tb.view(np.uint32))
    assert not np.array_equal(a[0], c[0])


# -- a K = 2, D = 8 swarm worked in exact rational arithmetic ------------------------------------
def test_tiny_swarm_by_exact_arithmetic(oracle):
    """Dyadic inputs, r from the big-integer Philox; every operation of
    Eq. (6), (7) done exactly and rounded once, as binary32 does."""
    K, D = 2, 8
    sixteenth = Fraction(1, 16)
    x0 = [[sixteenth * n for n in (3, -5, 8, 0, 12, -16, 1, 7)],
          [sixteenth * n for n in (-2, 4, 6, -9, 0, 5, -11, 13)]]
    v0 = [[sixteenth * n for n in (1, 0, -2, 3, -1, 4, 0, -3)],
          [sixteenth * n for n in (0, -1, 2, 2, -4, 1, 5, 0)]]
    p0 = [[sixteenth * n for n in (2, -4, 7, 1, 10, -12, 0, 6)],
          [sixteenth * n for n in (-1, 3, 8, -8, 1, 4, -10, 12)]]
    pl0, loss = [Fraction(1), Fraction(2)], [Fraction(3, 2), Fraction(5, 4)]
    # particle 1 has the lower loss (g = 1) and improves (5/4 < 2); particle 0 does not.
    w, c1, c2, seed, step = Fraction(1, 2), Fraction(1), Fraction(2), 20090003816, 7
    arr = lambda rows: np.array([[float(t) for t in r] for r in rows], F32)
    x, v, pbest = arr(x0), arr(v0), arr(p0)
    pl = np.array([float(t) for t in pl0], F32); ls = np.array([float(t) for t in loss], F32)
    gb = np.empty(D, F32)
    g, improved = oracle.sync(x, v, pbest, pl, ls, gb, F32(w), F32(c1), F32(c2), seed, step)
    assert g == 1 and improved.tolist() == [0, 1]
    assert pl.tolist() == [1.0, 1.25]
    p_new = [p0[0], x0[1]]
    for d in range(D):
        assert ef.frac(gb[d]) == x0[1][d]
        for i in range(K):
            r1, r2 = pb.draw_r_exact(seed, step, i, d)
            dp = ef.sub(p_new[i][d], x0[i][d]); dg = ef.sub(x0[1][d], x0[i][d])
            acc = ef.mul(w, v0[i][d])
            acc = ef.fma(ef.mul(c1, r1), dp, acc)
            acc = ef.fma(ef.mul(c2, r2), dg, acc)
            assert ef.frac(v[i, d]) == acc, (i, d)
            assert ef.frac(x[i, d]) == ef.add(x0[i][d], acc), (i, d)
            assert ef.frac(pbest[i, d]) == p_new[i][d]
