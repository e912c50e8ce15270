import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def _gpu_present() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _gpu_present():
        return
    skip = pytest.mark.skip(reason="no GPU in this container")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter, exitstatus, config):
    """How much of the GPU parity comparisons ran at the plain 1e-5 bound and how much of the
    forward-error allowance the rest used, per test (embedding tables / optimiser-state tables)."""
    from tests import parity_util
    stats = parity_util.STATS
    if not stats:
        return
    import json
    by_test = {}
    for st in stats:
        key = (st["test"].split("::", 1)[-1], st["kind"])
        a = by_test.setdefault(key, dict(n=0, inside=0.0, max_err_over_plain=0.0, allowance_used=0.0, dominant=0.0, untested=0.0))
        a["n"] += st["n"]
        a["inside"] += st["share_plain"] * st["n"]
        a["dominant"] += st["share_allowance_dominant"] * st["n"]
        a["untested"] += st["share_untested"] * st["n"]
        a["max_err_over_plain"] = max(a["max_err_over_plain"], st["max_err_over_plain"])
        a["allowance_used"] = max(a["allowance_used"], st["allowance_used"])
    tr = terminalreporter
    tr.section("parity comparisons: share at the plain bound, use of the forward-error allowance")
    tr.write_line(f"{'test':78s} {'table':5s} {'elements':>11s} {'at plain':>9s} {'max err/plain':>13s} {'allow. used':>11s} {'allow>plain':>11s} {'allow>lr':>9s}")
    rows = []
    for (test, kind), a in sorted(by_test.items()):
        n = max(a["n"], 1)
        row = dict(test=test, table=kind, elements=a["n"], share_plain=a["inside"] / n, max_err_over_plain=a["max_err_over_plain"],
                   allowance_used=a["allowance_used"], share_allowance_dominant=a["dominant"] / n, share_untested=a["untested"] / n)
        rows.append(row)
        tr.write_line(f"{test[:78]:78s} {kind:5s} {a['n']:11d} {row['share_plain']:9.5f} {row['max_err_over_plain']:13.2f} "
                      f"{row['allowance_used']:11.3f} {row['share_allowance_dominant']:11.4f} {row['share_untested']:9.2e}")
    out_dir = os.path.join(ROOT, "gpurun_out")
    if os.path.isdir(out_dir):
        with open(os.path.join(out_dir, "parity_stats.json"), "w") as fh:
            json.dump(rows, fh, indent=0)
