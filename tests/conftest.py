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


@pytest.fixture(autouse=True, scope="session")
def _workspace_guard():
    """GPU runs check, after every library call, a 16 MiB guard region behind the workspace the binding allocated:
    a kernel that writes past its workspace fails the test that made the call."""
    import torch
    if torch.cuda.is_available():
        import paper_1903_08114_amd as egp
        egp.set_workspace_guard(16 << 20)
    yield
