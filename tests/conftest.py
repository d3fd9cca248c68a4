import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped, not failed, on a machine without a GPU.
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture
def knobs():
    """Sets development knobs of the library (zipml_debug_set) for one test and restores the
    automatic choices afterwards."""
    from paper_1611_05402_amd import zipml
    used = []

    def set_knob(knob, value):
        zipml.debug_set(knob, value)
        used.append(knob)

    yield set_knob
    for knob in used:
        zipml.debug_set(knob, -1)
