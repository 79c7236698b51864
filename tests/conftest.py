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
    """Writes the parity errors measured in this session (tests/helpers.check_parity), largest first per dtype, to the
    file named by the environment variable QTALE_PARITY_REPORT."""
    try:
        from tests import helpers
    except Exception:
        return
    if not helpers.OBSERVED:
        return
    path = os.environ.get("QTALE_PARITY_REPORT")                # file to write; nothing is written without it
    if not path:
        return
    try:
        os.makedirs(os.path.dirname(os.path.abspath(path)), exist_ok=True)
        with open(path, "w") as f:
            for dt in ("bf16", "fp16"):
                rows = sorted((r for r in helpers.OBSERVED if r[1] == dt), key=lambda r: -r[2])
                if rows:
                    f.write("# %s: %d checks, max %.3e, contract %.0e\n" % (dt, len(rows), rows[0][2], helpers.TOL))
                    for what, _, err in rows[:40]:
                        f.write("%.3e  %s\n" % (err, what))
    except OSError:
        pass
