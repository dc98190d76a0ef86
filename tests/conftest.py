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
    """The built HIP library.  It is rebuilt here when it is missing or when the identifier it carries is not the
    hash of the present sources, header and flags, so a parity run never passes on a stale binary."""
    import paper_2602_09725_amd as kvc
    from paper_2602_09725_amd import build

    build.ensure_current()
    lib = kvc.load()
    assert lib.kvc_build_id().decode() == build.source_id()
    return lib
