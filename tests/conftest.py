import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    from tests import parity
    parity.set_pytest_config(config)


import pytest  # noqa: E402


@pytest.fixture(autouse=True)
def _gpu_tests_name_themselves(request):
    """A GPU test writes its name before it touches the device: a crash then names its case."""
    if request.node.get_closest_marker("gpu") is not None:
        from tests import parity
        parity.progress(f"\n[gpu test] {request.node.nodeid}")
    yield
