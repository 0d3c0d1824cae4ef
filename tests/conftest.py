import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_terminal_summary(terminalreporter):
    """Lists the errors the GPU parity checks observed (label, acceptance metric, worst and median per-row error),
    worst rows first, and keeps a copy next to the other outputs of a GPU run."""
    mod = sys.modules.get("paper_2503_06433_amd.harness")
    seen = getattr(mod, "OBSERVED", None) if mod else None
    if not seen:
        return
    lines = ["%-72s max|d|/max|ref| %.2e   row worst %.2e  median %.2e  (%d rows)" % rec
             for rec in sorted(seen, key=lambda r: -r[2])]
    terminalreporter.write_line("observed parity errors (%d checks), ten worst rows:" % len(lines))
    for ln in lines[:10]:
        terminalreporter.write_line("  " + ln)
    out_dir = os.path.join(ROOT, "gpurun_out")
    if os.path.isdir(out_dir):
        with open(os.path.join(out_dir, "parity_observed.txt"), "w") as f:
            f.write("\n".join(lines) + "\n")
