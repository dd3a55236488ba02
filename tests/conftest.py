import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs an MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def ngc():
    """The Python binding of libngc (argument marshalling only)."""
    from paper_2212_08580_amd import ngc as binding
    return binding


def parity_report(**figures):
    """Appends one JSON line of parity figures (worst and median errors, shares) to
    parity_report.jsonl in the directory NGC_REPORT_DIR names (default: test_reports/ beside
    tests/), so that they are kept with the test log instead of in a print that -q hides."""
    import json
    out_dir = os.environ.get("NGC_REPORT_DIR") or os.path.join(ROOT, "test_reports")
    try:
        os.makedirs(out_dir, exist_ok=True)
        with open(os.path.join(out_dir, "parity_report.jsonl"), "a") as f:
            f.write(json.dumps(figures) + "\n")
    except OSError:
        pass
