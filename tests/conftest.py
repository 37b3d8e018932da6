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
def canary_bands(request):
    """Every GPU test runs with canary bands in front of and behind each pool, staging and
    pinned-host buffer the harness allocates; a band that changed fails the test (pools closed
    inside the test are checked by close() itself)."""
    if request.node.get_closest_marker("gpu") is None:
        yield
        return
    from paper_2406_17565_amd.pool import TorchPool
    TorchPool.GUARD_BYTES = 1 << 20
    yield
    TorchPool.GUARD_BYTES = 0
    damaged = [p.geom for p in list(TorchPool.live) if not p.guards_intact()]
    assert not damaged, f"a copy wrote outside its buffer: pools with geometry {damaged}"
