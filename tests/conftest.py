import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _has_gpu():
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


@pytest.fixture
def progress(request):
    """Long tests say where they are on the real stdout (output capture is suspended for the line),
    so that whoever watches the run sees it advance during minutes of CPU-side oracle work."""
    capman = request.config.pluginmanager.getplugin("capturemanager")

    def say(msg):
        line = "\n[%s] %s" % (request.node.name, msg)
        if capman is None:
            print(line, flush=True)
            return
        with capman.global_and_fixture_disabled():
            print(line, flush=True)
    return say
