import os
import sys

import pytest

# every device allocation of the library gets guard zones that the fixture below checks after
# each GPU test (must be set before the library makes its first allocation)
os.environ.setdefault("LOP_GUARD_BYTES", "4096")

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import reference
    reference.build()
    return reference


@pytest.fixture(autouse=True)
def _no_store_outside_a_buffer(request):
    """After every GPU test: no kernel has stored outside a device allocation of the library."""
    yield
    if request.node.get_closest_marker("gpu") is None:
        return
    from paper_2507_05829_amd import lop
    assert lop.lop_debug_guard_check() == 0, "a kernel stored outside a device buffer (see stderr)"
