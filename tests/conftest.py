import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X")


@pytest.fixture(scope="session")
def orc32():
    from oracle import Oracle
    return Oracle("f32")


@pytest.fixture(scope="session")
def orc64():
    from oracle import Oracle
    return Oracle("f64")
