import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped (not failed) where no device is present, so that a plain
    # `pytest tests/` works on a CPU-only machine.
    try:
        import torch

        has_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this machine")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


class _Tuning:
    """Sets tuning switches of the library for one test (qnn_tuning_set) and restores the defaults."""

    def __init__(self):
        self._touched = set()

    def setenv(self, name, value):
        import paper_1806_08342_amd as qnn

        qnn.tuning_set(name, value)
        self._touched.add(name)

    def delenv(self, name, raising=False):
        import paper_1806_08342_amd as qnn

        qnn.tuning_set(name, None)

    def restore(self):
        import paper_1806_08342_amd as qnn

        for name in self._touched:
            qnn.tuning_set(name, None)


@pytest.fixture
def tuning():
    t = _Tuning()
    yield t
    t.restore()
