"""The library's host-side scalar helpers (Eq. (5), damping lambda, stage
cadence of Algorithm 1) against the oracle's.  No GPU needed."""
import numpy as np
import pytest

import paper_2009_03816_amd as pso

F32 = np.float32


def paper_settings():
    """tests/golden/paper_settings.txt: the constants of Table II and Section IV."""
    import os
    out = {}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_settings.txt")
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            key, *vals = line.split()
            out[key] = [float(v) for v in vals] if len(vals) > 1 else float(vals[0])
    return out


def test_paper_settings_give_the_papers_run_lengths(oracle):
    """With the printed settings: 234 iterations per MNIST epoch (60000/256), Max_t = 5850, a stage
    every 10th iteration -> 584 stages; inertia runs from just under 0.9 to 0.3 at Max_t; the
    damping takes c1 = 0.2 down to 0.2/25 in the last epoch."""
    ps = paper_settings()
    it = int(ps["mnist_training_size"] // ps["mnist_batch"])
    ep, step = int(ps["mnist_epochs"]), int(ps["mnist_step"])
    consts = tuple(F32(ps[k]) for k in ("m_max", "m_min", "c1", "c2"))
    assert (it, it * ep) == (234, 5850)
    flags = [pso.pso_ps_schedule(t, it, ep, step, *consts) for t in range(1, it * ep + 1)]
    assert sum(f[0] for f in flags) == 584
    assert F32(flags[-1][1]) == F32(0.3) and F32(0.8998) < F32(flags[0][1]) < F32(0.9)
    assert F32(flags[0][2]) == F32(0.2) and F32(flags[-1][2]) == F32(0.2) / F32(25)
    assert F32(flags[-1][3]) == F32(0.9) / F32(25)
    for t in (1, 234, 235, 5850):
        assert flags[t - 1][0] == oracle.schedule(t, it, ep, step, *consts)[0]
    it_c = int(ps["cifar_training_size"] // ps["cifar_batch"])
    assert it_c == 195 and pso.pso_ps_schedule(195 * 30, it_c, 30, 10, *consts)[0] is False


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
