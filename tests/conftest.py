import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def gpu_device():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


def pytest_sessionfinish(session, exitstatus):
    """PARITY_LOG=<file>: write looseness and containment of every GPU/oracle comparison of the session (one line each)."""
    path = os.environ.get("PARITY_LOG")
    if not path:
        return
    try:
        import parity
    except Exception:
        return
    with open(path, "w") as f:
        for what, loose, viol in parity.LOG:
            f.write(f"{loose:.4e}\t{viol:.4e}\t{what}\n")
