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


@pytest.fixture(autouse=True)
def _reset_tuning_switches():
    """Tests route calls to a kernel family with tsvd_tuning_set; every test starts from the library's own rules."""
    yield
    import paper_2308_07641_amd.tsvd as binding
    if binding._lib is not None:
        binding._lib.tsvd_tuning_reset()
