import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI library)")


def pytest_collection_modifyitems(config, items):
    import torch

    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


class _Options:
    """Sets switches of a context (pq_set_option) and returns them to their defaults afterwards."""

    def __init__(self, ctx):
        self.ctx, self.touched = ctx, set()

    def set(self, name, value):
        self.touched.add(name)
        self.ctx.pq_set_option(name, value)

    def restore(self):
        for name in self.touched:
            self.ctx.pq_set_option(name, None)


@pytest.fixture
def opts(ctx):
    o = _Options(ctx)
    yield o
    o.restore()
