import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture
def forced_plan():
    """Force the row sweep's launch shape ("threads,loads[,segments]") for the test, then hand it back to the library."""
    import paper_2505_13204_amd as aasd

    def force(shape: str):
        v = [int(x) for x in shape.split(",")]
        aasd.set_sweep_plan(v[0], v[1], v[2] if len(v) > 2 else 0)
    yield force
    aasd.set_sweep_plan(0, 0, 0)
