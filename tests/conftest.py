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
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture()
def knob():
    """Set library tuning knobs for one test (fc_tuning_set); every knob set is restored afterwards."""
    from paper_2505_21467_amd import binding as fc
    used = []

    def set_knob(name, value):
        fc.fc_tuning_set(name, value)
        used.append(name)

    yield set_knob
    for name in used:
        fc.fc_tuning_set(name, None)
