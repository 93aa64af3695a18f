import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


import pytest  # noqa: E402


@pytest.fixture(autouse=True)
def _gpu_tests_report_progress(request, capsys):
    """GPU tests write their name before they touch the device, and their progress lines as they go (not only when
    the test ends): a long oracle comparison is then visibly alive, and a crash names its case."""
    if request.node.get_closest_marker("gpu") is None:
        yield
        return
    with capsys.disabled():
        print(f"\n[gpu test] {request.node.nodeid}", flush=True)
        yield
