import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
# where GPU test runs leave what they measured (worst parity errors, progress of long oracle runs)
RUN_OUTPUT_DIR = os.path.join(ROOT, "gpurun_out")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def orc():
    import oracle
    oracle.build(force=False)
    return oracle


def pytest_sessionfinish(session, exitstatus):
    """GPU runs leave the worst relative error each parity assertion saw (by test and line)."""
    mod = sys.modules.get("gpu_util")
    if mod is None or not getattr(mod, "MEASURED", None):
        return
    import json
    out = RUN_OUTPUT_DIR
    os.makedirs(out, exist_ok=True)
    rows = sorted(({"file": k[0], "test": k[1], "line": k[2], "max_rel_l2": v} for k, v in mod.MEASURED.items()),
                  key=lambda r: (r["file"], r["line"]))
    with open(os.path.join(out, "measured_errors.json"), "w") as f:
        json.dump(rows, f, indent=1)
