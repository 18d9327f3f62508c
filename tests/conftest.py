import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def o32():
    import oracle
    return oracle.lib("f32")


@pytest.fixture(scope="session")
def o64():
    import oracle
    return oracle.lib("f64")
