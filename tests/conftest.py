import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


def pytest_sessionfinish(session, exitstatus):
    """After a GPU session: the errors the parity checks measured, next to the run's other
    outputs (only where that folder exists; a CPU-only session measures nothing)."""
    import json
    gpu_common = sys.modules.get("gpu_common")
    if gpu_common is None:
        return
    out_dir = os.path.join(ROOT, "gpurun_out")
    if not gpu_common.MEASURED or not os.path.isdir(out_dir):
        return
    rows = [dict(kind=k, what=w, **v) for (k, w), v in sorted(gpu_common.MEASURED.items())]
    with open(os.path.join(out_dir, "parity_measured.json"), "w") as f:
        json.dump(rows, f, indent=1)
