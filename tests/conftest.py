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
    """What the GPU parity run admitted beyond exact greedy ids, stated in the run's own output:
    every near-tie with the oracle's gap and the measured logit error that admitted it, and every
    activation comparison that exceeded the flat bar and was held to the oracle's own sensitivity."""
    util = sys.modules.get("tests.util")
    if util is None or not (util.ID_COMPARISONS[0] or util.BEYOND_FLAT):
        return
    tr = terminalreporter
    tr.write_line("")
    tr.write_line("parity summary: %d greedy-id comparisons, %d near-ties" % (util.ID_COMPARISONS[0], len(util.NEAR_TIES)))
    for line in util.NEAR_TIES:
        tr.write_line("  near-tie: " + line)
    tr.write_line("parity summary: %d comparisons beyond the flat bar, admitted by an oracle sensitivity run"
                  % len(util.BEYOND_FLAT))
    for line in util.BEYOND_FLAT:
        tr.write_line("  beyond flat: " + line)
