import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def c1():
    from workloads import make_config
    return make_config("c1_tiny")


@pytest.fixture(scope="session")
def c2():
    from workloads import make_config
    return make_config("c2_medium")


@pytest.fixture(scope="session")
def c3_graph():
    """The 10 M-state graph of configurations 3 and 4 (about 20 s to generate, 0.6 GB)."""
    from workloads.configs import make_graph
    return make_graph("c3_large")
