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
def opts():
    """Sets tuning overrides (ntp_set_option) on the default handle for one test and clears them afterwards."""
    import paper_2504_06095_amd as N
    touched = []

    def set_option(option, value):
        N.ntp_set_option(option, value)
        touched.append(option)

    yield set_option
    for option in touched:
        N.ntp_set_option(option, 0)
