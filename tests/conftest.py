import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "slow: long-running oracle comparison")


def pytest_collection_modifyitems(config, items):
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


@pytest.fixture(autouse=True)
def _progress(request):
    """Names each test on the real stderr as it starts and gives the helpers a `tick` that writes through pytest's
    capture: a long oracle comparison reports each layer it finishes instead of staying silent for minutes."""
    from tests import helpers
    capman = request.config.pluginmanager.getplugin("capturemanager")

    def tick(msg="."):
        with capman.global_and_fixture_disabled():
            sys.stderr.write(msg)
            sys.stderr.flush()

    helpers.tick = tick
    tick("\n[%s] " % request.node.name)
    yield
    helpers.tick = lambda msg=".": None
