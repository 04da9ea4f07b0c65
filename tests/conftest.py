import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _has_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


# Logits of a whole pass are held to the one-GEMV bar 2e-3 |W_row| |x| of the output head times this
# factor (bf16 roundings between the ops can fall differently in fp32 and fp64 and reach the head;
# the measured worst case over all logits tests is below a tenth of the bar).
LOGIT_SLACK = 1.0


def record_ratio(name: str, value: float) -> None:
    """Prints a measured error / tolerance ratio of a GPU parity test and, when the environment
    variable CAS_PARITY_RATIOS names a file, appends it there as a JSON line (the figures quoted
    in the design notes were collected that way)."""
    import json
    path = os.environ.get("CAS_PARITY_RATIOS")
    if path:
        try:
            with open(path, "a") as f:
                f.write(json.dumps({"test": name, "err_over_tol": float(value)}) + "\n")
        except OSError:
            pass
    print(f"[parity] {name}: err/tol = {value:.4g}", flush=True)
