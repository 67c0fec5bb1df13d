import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    """The CPU oracle (built on first use with the host compiler)."""
    from oracle import pso_ps_oracle
    pso_ps_oracle.build()
    return pso_ps_oracle


@pytest.fixture(params=["two_launches", "single_launch"])
def stage_launches(request, monkeypatch):
    """Runs a test twice: with every handle it creates told to take the stage
    in two launches, and in one (where the swarm is within the single-launch
    limit; larger ones keep the handle's default)."""
    import paper_2009_03816_amd as pso
    real_create = pso.pso_ps_create
    mode = 0 if request.param == "two_launches" else 1

    def create(K, *args, **kwargs):
        h = real_create(K, *args, **kwargs)
        if mode == 0 or K <= pso.PSO_PS_SINGLE_LAUNCH_MAX_K:
            pso.pso_ps_set_single_launch(h, mode)
        return h

    monkeypatch.setattr(pso, "pso_ps_create", create)
    return request.param
