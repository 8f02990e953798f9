import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # The shared library is a build product kept out of the history: load what is built, build only
    # if nothing is (hipcc cross-compiles for gfx950 without a GPU).
    from paper_2104_11981_amd import build as hip_build

    if not os.path.exists(hip_build.LIB):
        hip_build.build()


@pytest.fixture(scope="session")
def oracle():
    import oracle as _oracle

    _oracle.build()
    return _oracle
