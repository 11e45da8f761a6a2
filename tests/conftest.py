import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    import torch

    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


_observed = []  # (test id, what, kind, max abs, max row-relative)


@pytest.fixture(autouse=True)
def _collect_observed_errors(request):
    """Keeps the largest errors each parity test saw, so that the run's summary records the margins."""
    try:
        import parity
    except ImportError:
        yield
        return
    parity.OBSERVED.clear()
    yield
    worst = {}
    for what, kind, a, r in parity.OBSERVED:
        cur = worst.get(kind, (0.0, 0.0))
        worst[kind] = (max(cur[0], a), max(cur[1], r))
    for kind, (a, r) in worst.items():
        _observed.append((request.node.nodeid, kind, a, r))


def pytest_terminal_summary(terminalreporter):
    if not _observed:
        return
    terminalreporter.section("largest differences from the oracle, per test")
    for nodeid, kind, a, r in _observed:
        rel = f" row-rel {r:.2e}" if kind == "out" else ""
        terminalreporter.write_line(f"{nodeid}: {kind} max|d| {a:.2e}{rel}")
