import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI HIP library)")


@pytest.fixture
def plan_override():
    """Sets the library's launch-plan override for one test (the syntax of ATK_PLAN) and removes it afterwards."""
    import paper_2412_04358_amd as atk

    yield atk.set_plan_override
    atk.set_plan_override(None)
