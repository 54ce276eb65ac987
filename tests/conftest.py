import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped, loudly, where there is no GPU: a CPU fallback
    # would void every parity claim, so there is none.
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def pytest_terminal_summary(terminalreporter, exitstatus, config):
    """Near-threshold and in-band mismatch counts of every parity case that ran: printed in the
    summary (so they reach the log under -q as well) and kept as one JSON line per case."""
    try:
        import parity
    except Exception:
        return
    if not parity.REPORT:
        return
    import json
    tr = terminalreporter
    tr.section("parity: near-threshold nodes (exempt from bit-exactness) and nodes that differed")
    tot = {"nodes": 0, "near_threshold_draft": 0, "near_threshold_verify": 0, "mismatch_in_band": 0,
           "mismatch_in_band_stats": 0}
    lines = []
    for method, name, out in parity.REPORT:
        for key in tot:
            tot[key] += int(out.get(key, 0))
        lines.append(json.dumps({"method": method, "workload": name, **{k: (float(v) if isinstance(v, float) else int(v))
                                                                       for k, v in out.items()}}))
        tr.write_line("%-8s %-36s nodes %6d  near(draft) %4d  near(verify) %4d  differ %3d  differ(stats) %3d" % (
            method, name[:36], out.get("nodes", 0), out.get("near_threshold_draft", 0),
            out.get("near_threshold_verify", 0), out.get("mismatch_in_band", 0), out.get("mismatch_in_band_stats", 0)))
    tr.write_line("total: %s" % json.dumps(tot))
    try:
        d = os.path.join(ROOT, "gpurun_out")
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "parity_report.jsonl"), "w") as f:
            f.write("\n".join(lines) + "\n")
    except OSError:
        pass
