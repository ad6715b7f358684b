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
def tune():
    """``tune(pass_workers=3, ...)`` installs launch-shape overrides of the library for this test only."""
    import paper_2404_00438_amd as dl

    before = dl.dlion_get_tuning()

    def install(**fields):
        dl.dlion_set_tuning(dl.dlion_get_tuning(), **fields)

    yield install
    dl.dlion_set_tuning(before)
