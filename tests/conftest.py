import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
if os.path.dirname(os.path.abspath(__file__)) not in sys.path:
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are selected explicitly with -m gpu; without a visible device they are skipped.
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


class _Knobs:
    """Sets the library's tuning overrides (DSBD_* environment variables) for one test: the library reads them once
    per process, so every change is followed by a reload; on teardown the variables are removed and read again."""

    def __init__(self):
        self.names = []

    @staticmethod
    def _reload():
        import paper_2409_16560_amd as dsbd
        dsbd.dsbd_reload_knobs()

    def set(self, name, value):
        import os
        os.environ[name] = str(value)
        self.names.append(name)
        self._reload()

    def clear(self):
        import os
        for n in self.names:
            os.environ.pop(n, None)
        self.names = []
        self._reload()


@pytest.fixture
def knobs():
    k = _Knobs()
    try:
        yield k
    finally:
        k.clear()
