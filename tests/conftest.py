import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def gpu_up_before_inputs(request):
    """When GPU tests are selected, bring the device up before any test generates its inputs
    (input generation uses many host threads; the order init-then-generate is the one the
    benchmark uses too).  CPU-only sessions never touch the GPU runtime."""
    if any(item.get_closest_marker("gpu") for item in request.session.items):
        import torch
        if torch.cuda.is_available():
            torch.cuda.init()
            torch.ones(1, device="cuda:0").item()
    yield
