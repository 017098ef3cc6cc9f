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


# ---- parity report: worst errors of every oracle comparison, per test, at the end of a GPU run -------------
_PARITY = []


@pytest.fixture(autouse=True)
def _collect_parity(request):
    mod = sys.modules.get("gpu_util")
    if mod is not None:
        mod.WORST.clear()
    yield
    mod = sys.modules.get("gpu_util")
    if mod is not None and mod.WORST:
        _PARITY.append((request.node.nodeid, max(w[1] for w in mod.WORST), max(w[2] for w in mod.WORST),
                        len(mod.WORST)))
        mod.WORST.clear()


def pytest_terminal_summary(terminalreporter):
    if not _PARITY:
        return
    terminalreporter.section("oracle parity: worst max-abs / max-rel error per test")
    for nodeid, a, r, n in _PARITY:
        terminalreporter.write_line(f"{a:9.3e} {r:9.3e}  ({n:2d} comparisons)  {nodeid}")
