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
    from oracle import oracle as O
    O.build()
    return O


@pytest.fixture
def tune():
    """tune(option, value): set one of the library's test / tuning overrides (fs_tune_set) for
    the running test; every option touched goes back to automatic afterwards."""
    from paper_2201_00194_amd import api
    used = []

    def set_option(option, value):
        used.append(option)
        api.fs_tune_set(option, value)

    yield set_option
    for option in used:
        api.fs_tune_set(option, -1)
