import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run on the GPU box only)")


@pytest.fixture(scope="session")
def workloads():
    """Lazily built cache of the five synthetic workloads."""
    from paper_2304_14463_amd.inputs import make_workload
    cache = {}

    def get(cfg, B=None):
        key = (cfg, B)
        if key not in cache:
            cache[key] = make_workload(cfg, B)
        return cache[key]
    return get
