import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped (not failed) where no GPU exists and -m gpu was not asked for.
    try:
        import torch

        have_gpu = torch.cuda.is_available()
    except Exception:
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def pytest_sessionfinish(session, exitstatus):
    """Worst observed GPU-vs-oracle error per comparison label (digits and brackets stripped), for the record."""
    try:
        import json
        import re

        import parity

        if not parity.OBSERVED:
            return
        worst = {}
        for what, tol, e_inf, e_l2 in parity.OBSERVED:
            key = re.sub(r"\[[^\]]*\]|\d+", "", what).strip() or "unnamed"
            w = worst.setdefault(key, {"tol": tol, "max_rel": 0.0, "l2_rel": 0.0, "comparisons": 0})
            w["tol"] = max(w["tol"], tol)
            w["max_rel"] = max(w["max_rel"], e_inf)
            w["l2_rel"] = max(w["l2_rel"], e_l2)
            w["comparisons"] += 1
        out = os.path.join(ROOT, "gpurun_out")
        os.makedirs(out, exist_ok=True)
        with open(os.path.join(out, "parity_observed.json"), "w") as f:
            json.dump(worst, f, indent=1, sort_keys=True)
    except Exception:  # a record, never a reason to fail the run
        pass
