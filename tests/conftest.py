import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _gpu_available():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _gpu_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def pytest_terminal_summary(terminalreporter):
    """Largest observed errors of the floating-point comparisons, next to their bars."""
    try:
        import gpu_util
    except Exception:
        return
    for dt in ("bf16", "f32"):
        obs = [o for o in gpu_util.OBSERVED if o[0] == dt]
        if not obs:
            continue
        we = max(obs, key=lambda o: o[2])
        wr = max(obs, key=lambda o: o[3])
        terminalreporter.write_line(
            f"[parity {dt}] {len(obs)} comparisons; worst rel-Frobenius {we[2]:.3e} ({we[1]}) bar {gpu_util.TOL[dt]:g}; "
            f"worst row {wr[3]:.3e} ({wr[1]}) bar {gpu_util.ROW_TOL[dt]:g}")
