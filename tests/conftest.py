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
    from oracle import otf_oracle
    otf_oracle.build()
    return otf_oracle


@pytest.fixture
def debug_switches():
    """Sets diagnostic switches of the library for one test and clears them afterwards."""
    from paper_1407_4764_amd import binding
    used = []

    def set_all(switches):
        for key, value in switches.items():
            binding.debug_set(key, value)
            used.append(key)
    yield set_all
    for key in used:
        binding.debug_set(key, 0)
