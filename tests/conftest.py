import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """GPU tests fail loudly on a box with a GPU but no built library; on a box
    without a GPU they are skipped (they are deselected by -m "not gpu" anyway)."""
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    """What the GPU parity run admitted beyond the flat bars, stated in the run's own output: greedy-id
    near-ties (expected: none) and the comparisons whose absolute bound was scaled with the reference's
    magnitude (references beyond +-4)."""
    util = sys.modules.get("tests.util")
    if util is None or not (util.ID_COMPARISONS[0] or util.SCALED_BOUND_CASES):
        return
    tr = terminalreporter
    tr.write_line("")
    tr.write_line("parity summary: %d greedy-id comparisons, %d near-ties" % (util.ID_COMPARISONS[0], len(util.NEAR_TIES)))
    for line in util.NEAR_TIES:
        tr.write_line("  near-tie: " + line)
    tr.write_line("parity summary: %d comparisons used the scaled max-abs bound (reference beyond +-4)"
                  % len(util.SCALED_BOUND_CASES))
    for what, top, m, bound in util.SCALED_BOUND_CASES[:40]:
        tr.write_line("  scaled: %s: max|ref| %.2f, max abs err %.3e (bound %.3e)" % (what, top, m, bound))
