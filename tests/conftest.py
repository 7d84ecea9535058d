import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def zcref():
    """The reference CPU codec, built on demand with g++."""
    from oracle import zcref as z
    z.lib()
    return z


@pytest.fixture(params=["plain", "indexed"])
def stream_variant(request, zcref):
    """Runs a GPU test once per stream variant, with the library and the reference set alike."""
    import gpuutil
    gpuutil.set_variant(zcref, request.param == "indexed")
    yield request.param
    gpuutil.set_variant(zcref, False)
