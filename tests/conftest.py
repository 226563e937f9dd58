import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(params=["one_launch_where_allowed", "two_launches"])
def topk_path(request, monkeypatch):
    """SCORE + TOPK has a one-launch and a two-launch form with identical results; a call picks one by its
    shape.  Modules that use this fixture run every test under both, so that each form sees all their shapes."""
    import paper_2412_14468_amd as ha
    path = 2 if request.param == "one_launch_where_allowed" else 1
    orig = ha.Context.__init__

    def init(self, *a, **kw):
        orig(self, *a, **kw)
        self.hashattn_selftest_set_topk_path(path)
    monkeypatch.setattr(ha.Context, "__init__", init)
    return request.param
