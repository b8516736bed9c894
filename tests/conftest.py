import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture(scope="session", autouse=True)
def built_library():
    """The tests load the in-tree library; it is compiled here only if nothing has been built yet."""
    from paper_2506_22714_amd import binding as lb
    if not os.path.exists(lb.LIB_PATH):
        from paper_2506_22714_amd.build import build_library
        build_library()
    return lb.lib()
