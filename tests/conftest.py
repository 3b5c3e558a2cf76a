import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run on the GPU box)")


@pytest.fixture(scope="session")
def oracle_mod():
    import oracle
    # (tests/test_pins_catch_planted_mistakes.py runs the pins against other builds of the oracle)
    other = os.environ.get("DDEF_ORACLE_LIB")
    if other:
        oracle.use_library(other)
    oracle.build(force=False)
    return oracle
