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


def pytest_terminal_summary(terminalreporter, exitstatus, config):
    """Margins of the parity gate: for every test that compared against the oracle, the worst error under the
    asserted floor and under tighter ones (see tests/util.py).  Also written to the file named by the environment
    variable PARITY_MARGINS_OUT, if set."""
    try:
        from tests.util import MARGINS
    except Exception:
        return
    if not MARGINS:
        return
    cols = ["gate", "floor_S/16", "floor_S/64", "floor_1e-3_ref", "normwise_S", "normwise_ref"]
    lines = ["test | comparisons | asserted floor | " + " | ".join(cols)]
    for key in sorted(MARGINS):
        test, m = key[0], MARGINS[key]
        lines.append(f"{test} | {m['count']} | {m['floor']:.4g} | " + " | ".join(f"{m[c]:.3e}" for c in cols))
    terminalreporter.write_sep("-", "parity margins (worst per test)")
    for l in lines:
        terminalreporter.write_line(l)
    out = os.environ.get("PARITY_MARGINS_OUT")
    if out:
        with open(out, "w") as f:
            f.write("\n".join(lines) + "\n")
