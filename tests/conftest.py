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
    path = os.path.join(out_dir, "parity_measured.json")
    merged = {}
    if os.path.exists(path):                 # several pytest processes of one run add to one file
        try:
            merged = {(r["kind"], r["what"]): r for r in json.load(open(path))}
        except (ValueError, KeyError):
            merged = {}
    for (k, w), v in gpu_common.MEASURED.items():
        merged[(k, w)] = dict(kind=k, what=w, **v)
    with open(path, "w") as f:
        json.dump([merged[key] for key in sorted(merged)], f, indent=1)
