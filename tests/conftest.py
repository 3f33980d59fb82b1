import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def lib():
    """The loaded C-ABI library through the Python binding (GPU tests only)."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2510_12128_amd as pkg
    return pkg


def record_metric(name, **values):
    """Appends one line of measured parity numbers to parity_metrics.txt in the run-output
    folder (NUGPR_METRICS_DIR, else the folder below the repository root that GPU runs write
    to); kept for the results tables, ignored when the folder cannot be written."""
    try:
        out = os.environ.get("NUGPR_METRICS_DIR") or os.path.join(ROOT, "gpurun_out")
        os.makedirs(out, exist_ok=True)
        with open(os.path.join(out, "parity_metrics.txt"), "a") as f:
            f.write(name + " " + " ".join(f"{k}={v:.6e}" if isinstance(v, float) else f"{k}={v}"
                                           for k, v in values.items()) + "\n")
    except OSError:
        pass
