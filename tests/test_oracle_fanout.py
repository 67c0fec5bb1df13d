"""The column-range fan-out that the full-size GPU parity tests use to advance
the whole [K, D] state with the oracle: it must be the plain single-threaded
oracle call bit for bit (the update of a column never looks at another column;
the random numbers are indexed by the flat coordinate)."""
import numpy as np

from paper_2009_03816_amd import workloads as wl

import gpu_harness as gh

F32 = np.float32


def test_threaded_oracle_is_the_single_threaded_one(oracle):
    """The column-range fan-out used below, against one plain oracle call."""
    sw = wl.small_swarm(5, 20_001, seed=31, steps=2)
    one = [sw.x.copy(), sw.v.copy(), sw.pbest.copy(), sw.pbest_loss.copy(), np.zeros(20_001, F32)]
    fan = [a.copy() for a in one]
    gl1, gl2 = np.array([np.inf], F32), np.array([np.inf], F32)
    for s in range(2):
        r1 = oracle.sync(*one[:4], sw.losses[s], one[4], F32(0.7), F32(1.5), F32(1.5), 31, s,
                         gbest_loss=gl1)
        r2 = gh.oracle_sync_whole(oracle, *fan[:4], sw.losses[s], fan[4], 0.7, 1.5, 1.5, 31, s,
                                  gbest_loss=gl2)
        assert r1[0] == r2[0] and np.array_equal(r1[1], r2[1]) and r1[2] == r2[2]
        for a, b in zip(one + [gl1], fan + [gl2]):
            assert np.array_equal(gh.bits(a), gh.bits(b))
