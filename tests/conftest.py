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
def _library_knobs_follow_the_environment():
    """The library reads its PCCL_* switches when it is loaded; a test that changes one reloads
    them itself, and this re-reads them once the test (and monkeypatch's restore) is over."""
    yield
    from paper_2504_18658_amd import binding
    if binding._lib is not None:
        binding.diag_reload_env()
