"""Pins of the oracle's companions to the synchronization stage: historical
gBest (the standard-PSO reading of the global best), the scalar schedule
(Eq. (5), the damping lambda, Algorithm 1's cadence) and parameter averaging
(Section II-B, step 5)."""
from fractions import Fraction

import numpy as np
import pytest

import exact_fp32 as ef

F32 = np.float32


def swarm(rng, K, D):
    x = (rng.standard_normal((K, D)) * 0.05).astype(F32)
    v = (rng.standard_normal((K, D)) * 0.01).astype(F32)
    return x, v, x.copy(), np.full(K, np.inf, F32)


# ---------------------------------------------------------------- historical gBest
def test_history_first_stage_equals_memoryless(oracle):
    rng = np.random.default_rng(0)
    K, D = 5, 64
    x, v, p, pl = swarm(rng, K, D)
    loss = rng.uniform(0.1, 2, K).astype(F32)
    a = [t.copy() for t in (x, v, p, pl)] + [np.zeros(D, F32)]
    b = [t.copy() for t in (x, v, p, pl)] + [np.full(D, 9.0, F32)]
    ga, ia = oracle.sync(*a[:4], loss, a[4], F32(0.7), F32(1.5), F32(1.5), 3, 0)
    gl = np.array([np.inf], F32)
    gb, ib, rep = oracle.sync(*b[:4], loss, b[4], F32(0.7), F32(1.5), F32(1.5), 3, 0, gbest_loss=gl)
    assert rep and ga == gb and np.array_equal(ia, ib) and gl[0] == loss.min()
    for ta, tb in zip(a, b):
        assert np.array_equal(ta.view(np.uint32), tb.view(np.uint32))


def test_history_is_the_first_best_of_all_stages(oracle):
    """Brute force: keep every pre-move position; gbest must be the position
    of the earliest, lowest-index occurrence of the lowest loss so far."""
    rng = np.random.default_rng(1)
    K, D, steps = 4, 33, 25
    x, v, p, pl = swarm(rng, K, D)
    gbest, gl = np.full(D, np.nan, F32), np.array([np.inf], F32)
    losses = rng.uniform(0.1, 2.5, (steps, K)).astype(F32)
    losses[7] = 2.4; losses[7, 1] = losses[:7].min()   # ties the best so far: no replacement
    losses[12, 2] = np.nan
    snapshots, n_replaced = [], 0
    for s in range(steps):
        snapshots.append(x.copy())
        prev_bits, prev_gl = gbest.view(np.uint32).copy(), gl[0]
        g, improved, rep = oracle.sync(x, v, p, pl, losses[s], gbest, F32(0.6), F32(0.5), F32(0.5),
                                       11, s, gbest_loss=gl)
        hist = np.where(np.isnan(losses[:s + 1]), np.inf, losses[:s + 1])
        s_best, g_best = np.unravel_index(np.argmin(hist), hist.shape)   # first occurrence
        assert gl[0] == hist.min() and gl[0] <= prev_gl
        assert np.array_equal(gbest.view(np.uint32), snapshots[s_best][g_best].view(np.uint32))
        assert rep == (s_best == s)
        if not rep:
            assert np.array_equal(gbest.view(np.uint32), prev_bits)
        n_replaced += rep
        assert g == int(np.argmin(np.where(np.isnan(losses[s]), np.inf, losses[s])))
    assert 2 <= n_replaced < steps and losses[7].min() == losses[:7].min()


def test_history_move_uses_the_kept_gbest(oracle):
    """In a stage that does not replace gbest, Eq. (6) pulls towards the old
    gbest, also for this stage's best particle."""
    rng = np.random.default_rng(2)
    K, D = 3, 200
    x, v, p, pl = swarm(rng, K, D)
    pl[:] = 0.0                                # nobody improves: pbest stays
    p += F32(0.01)
    gbest = (rng.standard_normal(D) * 0.05).astype(F32)
    keep = gbest.copy()
    gl = np.array([0.05], F32)
    loss = np.array([0.9, 0.3, 0.6], F32)      # min 0.3 > 0.05: no replacement
    x0, v0 = x.astype(np.float64), v.astype(np.float64)
    g, improved, rep = oracle.sync(x, v, p, pl, loss, gbest, F32(0.7), F32(0.4), F32(0.8), 5, 9,
                                   gbest_loss=gl)
    assert g == 1 and not rep and not improved.any() and gl[0] == F32(0.05)
    assert np.array_equal(gbest, keep)
    r = np.array([[oracle.draw_r(5, 9, i, d) for d in range(D)] for i in range(K)], np.float64)
    t0 = float(F32(0.7)) * v0
    t1 = float(F32(0.4)) * r[..., 0] * (p.astype(np.float64) - x0)
    t2 = float(F32(0.8)) * r[..., 1] * (keep.astype(np.float64)[None, :] - x0)
    mag = np.abs(t0) + np.abs(t1) + np.abs(t2)
    assert np.all(np.abs(v.astype(np.float64) - (t0 + t1 + t2)) <= 3 * 2.0 ** -24 * mag + 1e-45)
    assert np.abs(t2[1]).max() > 1e-4          # the best particle does feel the old gbest


def test_history_all_nan_keeps_gbest(oracle):
    rng = np.random.default_rng(3)
    x, v, p, pl = swarm(rng, 3, 10)
    gbest, gl = np.arange(10, dtype=F32), np.array([np.inf], F32)
    g, improved, rep = oracle.sync(x, v, p, pl, np.full(3, np.nan, F32), gbest, F32(0.5), F32(1),
                                   F32(1), 0, 0, gbest_loss=gl)
    assert g == 0 and not rep and np.isinf(gl[0]) and np.array_equal(gbest, np.arange(10, dtype=F32))


# ---------------------------------------------------------------- Eq. (5), lambda, cadence
def test_inertia_endpoints_line_and_table2(oracle):
    m_max, m_min = F32(0.9), F32(0.3)          # Table II
    assert oracle.inertia(0, 1000, m_max, m_min) == m_max
    assert oracle.inertia(1000, 1000, m_max, m_min) == m_min
    t_max = 5850                               # 25 epochs of 234 iterations
    vals = [oracle.inertia(t, t_max, m_max, m_min) for t in range(t_max + 1)]
    assert all(a >= b for a, b in zip(vals, vals[1:])) and vals[0] > vals[-1]
    for t in (1, 2, 17, 2925, 5849):
        exact = Fraction(float(m_max)) - t * (Fraction(float(m_max)) - Fraction(float(m_min))) / t_max
        assert abs(Fraction(float(vals[t])) - exact) <= abs(exact) * Fraction(1, 1 << 24) * Fraction(1001, 1000)
    assert abs(float(vals[2925]) - 0.6) < 1e-7


def test_schedule_cadence_lambda_and_damping(oracle):
    it, ep, step = 234, 25, 10                 # MNIST runs: 60000/256 iterations, 25 epochs, step 10
    max_t = it * ep
    stages, lambdas = 0, set()
    for t in range(1, max_t + 1):
        is_stage, w, a1, a2 = oracle.schedule(t, it, ep, step, F32(0.9), F32(0.3), F32(0.2), F32(0.9))
        lam = (t - 1) // it + 1
        lambdas.add(lam)
        assert is_stage == (t % step == 0 and t < max_t)
        stages += is_stage
        assert w == oracle.inertia(t, max_t, F32(0.9), F32(0.3))
        assert ef.frac(a1) == ef.rnd(ef.frac(F32(0.2)) / lam)      # one correctly rounded division
        assert ef.frac(a2) == ef.rnd(ef.frac(F32(0.9)) / lam)
    assert stages == (max_t - 1) // step and lambdas == set(range(1, ep + 1))
    for bad in [(0, it, ep, step), (max_t + 1, it, ep, step), (1, 0, ep, step), (1, it, 0, step),
                (1, it, ep, 0)]:
        with pytest.raises(ValueError):
            oracle.schedule(*bad, F32(0.9), F32(0.3), F32(0.2), F32(0.9))


# ---------------------------------------------------------------- parameter averaging
def test_average_exact_rational_and_rows(oracle):
    rng = np.random.default_rng(4)
    for K in (1, 2, 3, 7, 16):
        D = 40
        x = (rng.standard_normal((K, D)) * 0.05).astype(F32)
        x0 = x.copy()
        mean = np.empty(D, F32)
        oracle.average(x, mean)
        for d in range(D):
            acc = ef.frac(x0[0, d])
            for k in range(1, K):
                acc = ef.add(acc, ef.frac(x0[k, d]))
            assert ef.frac(mean[d]) == ef.rnd(acc / K), (K, d)
        assert all(np.array_equal(x[k].view(np.uint32), mean.view(np.uint32)) for k in range(K))
        true = x0.astype(np.float64).mean(axis=0)
        assert np.all(np.abs(mean - true) <= K * 2.0 ** -24 * np.abs(x0).astype(np.float64).max(axis=0))


def test_average_special_cases(oracle):
    row = np.array([0.1, -2.5, 3.0, 1e-30, 0.0], F32)
    x = np.tile(row, (2, 1)); mean = np.empty(5, F32)
    oracle.average(x, mean)
    assert np.array_equal(mean, row)                       # (a + a) / 2 == a exactly
    x = np.array([[1, 2, 3], [3, 2, 1], [2, 2, 2], [6, 2, -6]], F32)
    mean = np.empty(3, F32); oracle.average(x, mean)
    assert mean.tolist() == [3.0, 2.0, 0.0]
    pad = np.full((3, 8), 7.0, F32); pad[:, :5] = np.arange(15, dtype=F32).reshape(3, 5)
    mean = np.empty(5, F32); oracle.average(pad[:, :5], mean)
    assert mean.tolist() == [5.0, 6.0, 7.0, 8.0, 9.0] and np.all(pad[:, 5:] == 7.0)
