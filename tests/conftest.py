import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # A GPU test must never silently pass on a box without a GPU.
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    """How often a bf16 comparison needed the half-ulp allowance beyond 5 RMS (helpers.assert_close)."""
    try:
        import helpers
    except Exception:  # pragma: no cover
        return
    if not helpers.tail_log:
        return
    tot = len(helpers.tail_log)
    elems = sum(n for _, n, _, _ in helpers.tail_log)
    tail = sum(t for _, _, t, _ in helpers.tail_log)
    used = [(w, u) for w, _, _, u in helpers.tail_log if u]
    terminalreporter.write_line(
        f"parity bar: {tot} bf16 tensors compared, {elems} elements, {tail} of them beyond 5 RMS; "
        f"{sum(u for _, u in used)} elements of {len(used)} tensors needed the half-ulp allowance")
    for w, u in used[:40]:
        terminalreporter.write_line(f"  half-ulp allowance used: {w}: {u} element(s)")
