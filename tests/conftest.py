import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_report_header(config):
    """Which HIP library this run loads: its hash, and a warning if a source is newer than it."""
    import hashlib
    from paper_2504_14960_amd.build import LIB, stale_sources
    if not os.path.exists(LIB):
        return "libmoe_hip.so: MISSING (python -m paper_2504_14960_amd.build)"
    digest = hashlib.sha256(open(LIB, "rb").read()).hexdigest()[:16]
    stale = stale_sources()
    note = f"  STALE: newer sources {stale}" if stale else "  (up to date with csrc/)"
    return f"libmoe_hip.so sha256 {digest}{note}"


def _have_gpu() -> bool:
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
