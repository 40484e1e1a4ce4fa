import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped, not failed, where no GPU is visible."""
    import torch
    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_sessionfinish(session, exitstatus):
    """Write the worst observed err/floor of every gap-vector comparison (tests/gpu_common.py) to
    gpurun_out/tolerance_margins.txt, so the margins of the per-entry fp32 floor can be read after a run."""
    mod = sys.modules.get("gpu_common")
    margins = getattr(mod, "MARGINS", None) if mod else None
    if not margins:
        return
    out = os.path.join(ROOT, "gpurun_out")
    os.makedirs(out, exist_ok=True)
    with open(os.path.join(out, "tolerance_margins.txt"), "w") as f:
        f.write("label | worst err/floor | most entries that needed the floor | comparisons\n")
        for label in sorted(margins):
            worst, needed, count = margins[label]
            f.write(f"{label} | {worst:.3f} | {needed} | {count}\n")
