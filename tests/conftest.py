import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _have_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _have_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


@pytest.fixture
def launch_knobs():
    """Setter for the library's launch-geometry knobs that puts every knob back to 0 (the library's own choice)
    when the test ends."""
    from paper_2205_13104_amd import binding as twa
    touched = set()

    def set_knob(knob, value):
        touched.add(knob)
        twa.set_launch_knob(knob, value)

    yield set_knob
    for knob in touched:
        twa.set_launch_knob(knob, 0)
