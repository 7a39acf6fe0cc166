import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _asks_for_gpu(config) -> bool:
    """True when the -m expression selects the gpu marker itself (not its negation)."""
    expr = (config.getoption("-m") or "").strip()
    return "gpu" in expr and "not gpu" not in expr


def pytest_collection_modifyitems(config, items):
    # Without a device, GPU tests of an unfiltered run are skipped; a run that asked for
    # them with -m gpu fails instead: a box whose GPU did not come up must not read as green.
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        has_gpu = False
    if has_gpu:
        return
    if _asks_for_gpu(config) and any("gpu" in item.keywords for item in items):
        pytest.exit("-m gpu was requested but torch.cuda.is_available() is False", returncode=3)
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
