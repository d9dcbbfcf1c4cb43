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


@pytest.fixture(scope="session", autouse=True)
def parity_error_report():
    """Writes the errors the GPU parity tests achieved (tests/harness.py: record) to parity_errors.json in the directory
    TEAM_MOE_REPORT_DIR names (default: test_reports/ at the repository root)."""
    yield
    try:
        import harness
    except Exception:
        return
    if harness.RECORDS:
        import json
        out = os.environ.get("TEAM_MOE_REPORT_DIR") or os.path.join(ROOT, "test_reports")
        os.makedirs(out, exist_ok=True)
        with open(os.path.join(out, "parity_errors.json"), "w") as f:
            json.dump({"row_rel": "per row max|gpu-ref| / max|ref|, max over rows", "elem": "max |gpu-ref| / max(|ref|, 1e-3 rms(ref))",
                       "cases": harness.RECORDS}, f, indent=1, sort_keys=True)
