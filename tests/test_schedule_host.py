"""The library's host-side scalar helpers (Eq. (5), damping lambda, stage
cadence of Algorithm 1) against the oracle's.  No GPU needed."""
import numpy as np
import pytest

import paper_2009_03816_amd as pso

F32 = np.float32


def test_inertia_matches_oracle(oracle):
    rng = np.random.default_rng(0)
    for _ in range(3000):
        t_max = int(rng.integers(1, 10 ** 7))
        t = int(rng.integers(0, t_max + 1))
        m_min, m_max = sorted(rng.uniform(0, 2, 2).astype(F32))
        assert F32(pso.pso_ps_inertia(t, t_max, m_max, m_min)) == oracle.inertia(t, t_max, m_max, m_min)
    assert F32(pso.pso_ps_inertia(0, 50, 0.9, 0.3)) == F32(0.9)
    assert F32(pso.pso_ps_inertia(50, 50, 0.9, 0.3)) == F32(0.3)


def test_schedule_matches_oracle_over_a_whole_run(oracle):
    it, ep, step = 234, 25, 10                      # the paper's MNIST settings with Table II
    args = (F32(0.9), F32(0.3), F32(0.2), F32(0.9))
    for t in range(1, it * ep + 1):
        got = pso.pso_ps_schedule(t, it, ep, step, *args)
        want = oracle.schedule(t, it, ep, step, *args)
        assert got[0] == want[0] and all(F32(a) == b for a, b in zip(got[1:], want[1:])), t
    for bad in [(0, it, ep, step), (it * ep + 1, it, ep, step), (1, 0, ep, step), (1, it, 0, step),
                (1, it, ep, 0), (1, 2 ** 40, 2 ** 40, 1)]:
        with pytest.raises(pso.PsoPsError) as e:
            pso.pso_ps_schedule(*bad, *args)
        assert e.value.code == pso.PSO_PS_EINVAL
