import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # GPU tests are skipped automatically where no GPU is visible.
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_sessionfinish(session, exitstatus):
    """Writes the parity errors measured in this session (tests/helpers.check_parity), largest first per dtype."""
    try:
        from tests import helpers
    except Exception:
        return
    if not helpers.OBSERVED:
        return
    out_dir = os.path.join(ROOT, "gpurun_out")
    try:
        os.makedirs(out_dir, exist_ok=True)
        with open(os.path.join(out_dir, "parity_errors.txt"), "w") as f:
            for dt in ("bf16", "fp16"):
                rows = sorted((r for r in helpers.OBSERVED if r[1] == dt), key=lambda r: -r[2])
                if rows:
                    f.write("# %s: %d checks, max %.3e, contract %.0e\n" % (dt, len(rows), rows[0][2], helpers.TOL))
                    for what, _, err in rows[:40]:
                        f.write("%.3e  %s\n" % (err, what))
    except OSError:
        pass
