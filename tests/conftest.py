import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


# compiled kernels of a test session go to a private directory, not to ~/.cache
_CACHE = os.path.join(ROOT, ".pytest_cache", "grumpy_hip_kernels")
os.makedirs(_CACHE, exist_ok=True)
os.environ.setdefault("GR_CACHE_DIR", _CACHE)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped, not failed, where no device is visible.
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    # how many elements of each reduction comparison passed the strict per-element bar and how many
    # only the bar against the caller's cancellation scale (sum|terms|)
    try:
        from helpers import SCALE_REPORT
    except Exception:
        return
    if not SCALE_REPORT:
        return
    total = sum(n for _, n, _ in SCALE_REPORT)
    needed = sum(k for _, _, k in SCALE_REPORT)
    terminalreporter.write_line(f"reduction comparisons: {len(SCALE_REPORT)} arrays, {total} elements, "
                                f"{total - needed} within 1e-5 of the oracle per element, {needed} only within 1e-5 of sum|terms|")
    for what, n, k in SCALE_REPORT:
        if k:
            terminalreporter.write_line(f"  {what}: {k} of {n} needed the cancellation scale")
