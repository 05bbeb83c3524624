import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _has_gpu() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture
def tuning():
    """Set tuning knobs of the library for one test (mole_set_tuning); every knob set is restored to the
    library's own choice afterwards."""
    from paper_2503_15798_amd import binding as mb
    touched = []

    def set_knob(name, value):
        mb.mole_set_tuning(name, int(value))
        touched.append(name)
    yield set_knob
    for name in touched:
        mb.mole_set_tuning(name, 0)
