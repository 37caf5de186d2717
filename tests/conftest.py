import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "slow: long-running CPU test")


def _has_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


@pytest.fixture(autouse=True)
def _poisoned_workspaces(monkeypatch):
    """Every workspace the tests hand to the library starts as NaN bit patterns (0xFF bytes): a kernel that reads
    scratch memory it has not written (padding columns, stale tables) turns the output into NaN instead of passing
    on whatever the allocator happened to return."""
    if not _has_gpu():
        yield
        return
    import torch
    from paper_2603_26498_amd import runtime

    def poisoned(self, nbytes):
        t = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)
        t.fill_(0xFF)
        return t

    monkeypatch.setattr(runtime.VisionEncoder, "workspace", poisoned)
    yield
