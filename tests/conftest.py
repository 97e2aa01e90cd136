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
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    """worst tau / s_local relative error against the oracle seen by the GPU parity tests"""
    worst = getattr(sys.modules.get("parity_util"), "WORST", None)
    if worst:
        terminalreporter.write_sep("-", "worst relative error of the statistics vs the oracle (bound: 1e-6)")
        for what in sorted(worst):
            terminalreporter.write_line("%-40s %.3e" % (what, worst[what]))


@pytest.fixture(scope="session")
def oracle():
    import oracle as o
    o.build()
    o.lib()
    return o
