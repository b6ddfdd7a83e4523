import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    import torch
    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


class _Options:
    """Sets the library's implementation switches for one test; the values it gives
    may be strings of digits, as an environment variable would hold them."""

    def __init__(self):
        from paper_2409_04992_amd import binding
        self._binding = binding

    def setenv(self, name, value):
        self._binding.set_option(name, int(value))

    def delenv(self, name, raising=True):
        self._binding.set_option(name, None)

    def reset(self):
        for name in self._binding.OPTIONS:
            self._binding.set_option(name, None)


@pytest.fixture
def options():
    """The library's switches, all handed back to the host before and after the test."""
    o = _Options()
    o.reset()
    yield o
    o.reset()
