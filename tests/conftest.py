import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def load_golden(name):
    """Parse a tests/golden/*.txt fixture: '#' lines are comments (the citation), other
    lines are 'key: v0 v1 ...' with float values."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, vals = line.split(":", 1)
            out[key.strip()] = [float(v) for v in vals.split()]
    return out


@pytest.fixture
def golden():
    return load_golden


def pytest_terminal_summary(terminalreporter):
    """Largest element-wise error ratio seen per mixed-precision check (tests/harness.py: check_bf16_tensor)."""
    try:
        import harness
    except Exception:
        return
    if harness.observed_elem_err:
        worst = sorted(harness.observed_elem_err.items(), key=lambda kv: -kv[1])[:12]
        terminalreporter.write_line("largest element-wise bf16 error ratios: " + ", ".join(f"{k}={v:.3f}" for k, v in worst))
