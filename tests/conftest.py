import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


import pytest


@pytest.fixture(autouse=True)
def _guard_bytes_untouched(request):
    """After every GPU test: the guard elements around the buffers the helpers allocated are intact."""
    yield
    if request.node.get_closest_marker("gpu") is not None:
        import gpu_util
        gpu_util.check_guards()
