import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def _have_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _have_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_terminal_summary(terminalreporter, exitstatus, config):
    """Per-case parity figures of the GPU tests (relative L2 error of gradients / weights against the oracle)."""
    try:
        from tests.gpu_util import PARITY
    except Exception:
        return
    if not PARITY:
        return
    tr = terminalreporter
    tr.write_line("")
    tr.write_line("parity summary: worst per-tensor relative L2 error, its tensor (median over tensors) [tensors above 2e-2]")
    fmt = lambda x: f"{x['worst']:.4f} {x['worst_tensor']} ({x['median']:.4f}) [{len(x['above_2e-2'])}]"
    for r in PARITY:
        line = f"  {r['case']}: {fmt(r['asserted'])}"
        for label, x in r.items():
            if isinstance(x, dict) and label != "asserted":
                line += f" | {label}: {fmt(x)}"
        if r.get("note"):
            line += f" | {r['note']}"
        tr.write_line(line)
    try:
        import json
        out = os.environ.get("NMT_TEST_OUTPUT_DIR") or os.path.join(ROOT, "gpurun_out")
        os.makedirs(out, exist_ok=True)
        with open(os.path.join(out, "parity_summary.json"), "w") as f:
            json.dump(PARITY, f, indent=1)
    except OSError:
        pass
