import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # every gpu-marked test is skipped outright when no device is visible
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:  # pragma: no cover
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter, exitstatus, config):
    """Totals of the parity comparisons of this run: evaluations compared, best-response
    mismatches by class, and how often the sweep's winner was the oracle's own."""
    try:
        from tests import parity
    except Exception:  # pragma: no cover
        return
    ev = [r for r in parity.LOG if r["kind"] == "eval"]
    wn = [r for r in parity.LOG if r["kind"] == "winner"]
    if not ev and not wn:
        return
    tot = {k: sum(r[k] for r in ev) for k in ("n_evals", "br_mismatch", "flagged", "bound_explained", "hard")}
    terminalreporter.write_line(
        "parity totals: %d comparisons, %d evaluations, %d best-response mismatches "
        "(%d flagged gap<1e-6*s, %d bound-explained, %d hard); winner index equal to the oracle's in "
        "%d of %d sweeps" % (len(ev), tot["n_evals"], tot["br_mismatch"], tot["flagged"],
                              tot["bound_explained"], tot["hard"],
                              sum(r["same_index"] for r in wn), len(wn)))
    out = os.environ.get("BSSE_PARITY_LOG")          # a file to keep the counts in, if asked for
    if out:
        import json
        with open(out, "w") as f:
            json.dump({"totals": tot, "winner_checks": len(wn),
                       "winner_same_index": sum(r["same_index"] for r in wn), "log": parity.LOG}, f)
