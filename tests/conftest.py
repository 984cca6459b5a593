import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped (not failed) when no device is visible, e.g. when the
    # whole suite is run without -m on a CPU-only machine.
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


class _Options:
    """Sets tuning options of the library for one test and restores the defaults afterwards."""

    def __init__(self):
        self.touched = set()

    def set(self, name, value):
        """name: the option's name (an "NQ_" prefix and capitals are accepted); value: int, its decimal
        string, or None for the default."""
        from paper_2602_06694_amd import binding as nq
        name = name[3:].lower() if name.startswith("NQ_") else name
        nq.nq_set_option(name, None if value is None else int(value))
        self.touched.add(name)

    def unset(self, name):
        self.set(name, None)

    def restore(self):
        from paper_2602_06694_amd import binding as nq
        for name in self.touched:
            nq.nq_set_option(name, None)


@pytest.fixture
def nqopt():
    o = _Options()
    yield o
    o.restore()
