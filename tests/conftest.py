import os
import shutil
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI library)")


@pytest.fixture(autouse=True)
def _remove_tier_files_after_the_test(request):
    """File-tier tests write tens of GiB under tmp_path, which pytest keeps until the session ends;
    the tests that size themselves by the free disk space (configurations 4 and 5 at the depth the
    box holds) come last and must find the disk as empty as a benchmark run does."""
    path = str(request.getfixturevalue("tmp_path")) if "tmp_path" in request.fixturenames else None
    yield
    if path:
        shutil.rmtree(path, ignore_errors=True)
