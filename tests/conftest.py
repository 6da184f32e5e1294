import os
import sys

import pytest

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(autouse=True)
def _guard_bands_intact(request):
    """After every GPU test: no kernel wrote outside a guarded output or workspace."""
    yield
    if request.node.get_closest_marker("gpu") is not None:
        dev = sys.modules.get("tests.device")
        if dev is not None:
            dev.check_all_guards()
