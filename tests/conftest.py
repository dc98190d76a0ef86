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
    from oracle import kvco_py

    kvco_py.lib()
    return kvco_py


@pytest.fixture(scope="session")
def kvc_lib():
    """The built HIP library; built here only if no build is present."""
    import paper_2602_09725_amd as kvc

    if not os.path.exists(kvc.lib_path()):
        from paper_2602_09725_amd import build

        build.build()
    return kvc.load()
