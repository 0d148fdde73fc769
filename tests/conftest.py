import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _built_library():
    """The tests load the in-tree library; it is compiled here only when nothing has been built yet."""
    from paper_2306_01381_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2306_01381_amd.build import build_library
        build_library(verbose=False)


@pytest.fixture(scope="session")
def oracle():
    import oracle as _oracle
    _oracle.lib()
    return _oracle
