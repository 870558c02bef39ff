import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "slow: full-size configuration")


@pytest.fixture(scope="session")
def configs_small():
    """TAS of configurations 0-2 (cheap to build), built once per session."""
    from workloads import make_tas
    return {i: make_tas(i) for i in range(3)}


@pytest.fixture
def tuning():
    """Forces launch choices of the library for one test (tensile_tuning_set) and puts the automatic ones back."""
    import paper_2105_13336_amd as P
    yield P.tensile_tuning_set
    P.tensile_tuning_reset()
