import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def built_library():
    """The tests load the library that is built; they build it only if nothing is."""
    from paper_2001_05585_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.LIB_PATH


@pytest.fixture(scope="session")
def oracle_lib():
    import oracle
    oracle.build(force=False)
    return oracle
