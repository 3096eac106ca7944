import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def oracle_mod():
    """The CPU oracle, compiled on first use."""
    import oracle
    oracle._load()
    return oracle


@pytest.fixture(autouse=True)
def _dirty_workspaces(request, monkeypatch):
    """GPU tests: every workspace the binding allocates itself starts as all-ones bytes (NaN as floats,
    -1 as integers), so that a kernel relying on what a workspace held before its call shows."""
    if request.node.get_closest_marker("gpu") is None:
        yield
        return
    from paper_2308_03291_amd import binding
    plain = binding._workspace

    def dirty(op, B, N, T, dt, device, workspace):
        ws, n = plain(op, B, N, T, dt, device, workspace)
        if workspace is None:
            ws.fill_(0xFF)
        return ws, n

    monkeypatch.setattr(binding, "_workspace", dirty)
    yield
