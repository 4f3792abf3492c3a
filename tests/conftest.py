import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped (not failed) when no device is present."""
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_sessionfinish(session, exitstatus):
    """The plain error figures the GPU parity tests saw, per tensor, for the record (gpurun_out/ is the
    folder that comes back from a GPU run)."""
    try:
        from tests import test_gpu_parity as tp
    except Exception:
        return
    if not tp.OBSERVED:
        return
    out = os.path.join(ROOT, "gpurun_out")
    try:
        os.makedirs(out, exist_ok=True)
        worst = {}
        for name, rel, mabs, big in tp.OBSERVED:
            w = worst.setdefault(name, [0.0, 0.0, 0.0, 0])
            w[0], w[1], w[2], w[3] = max(w[0], rel), max(w[1], mabs), max(w[2], big), w[3] + 1
        with open(os.path.join(out, "parity_observed.txt"), "w") as f:
            f.write("tensor  comparisons  worst rel-L2  worst max-abs error  largest |reference|\n")
            for name, (rel, mabs, big, n) in sorted(worst.items()):
                f.write(f"{name:6s} {n:5d}  {rel:.3e}  {mabs:.3e}  {big:.3e}\n")
    except OSError:
        pass
