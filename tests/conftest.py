import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def repo_root():
    return ROOT


def pytest_terminal_summary(terminalreporter):
    """Achieved errors of the GPU comparisons, largest per test function."""
    from tests import gpu_util
    if not gpu_util.ERROR_REPORT:
        return
    worst = {}
    for test, row in gpu_util.ERROR_REPORT.items():
        name = test.split("[", 1)[0]
        w = worst.setdefault(name, {"err": 0.0, "rel": 0.0, "tight": 0.0, "lse": 0.0, "n": 0})
        for k in ("err", "rel", "tight", "lse"):
            w[k] = max(w[k], row[k])
        w["n"] += 1
    tr = terminalreporter
    tr.write_sep("-", "GPU against the float64 oracle: largest errors per test (gate: |err| <= 1e-2 + 1e-2 |ref|)")
    tr.write_line("(max|err| is mostly the bf16 rounding of the largest outputs; /derived: largest |err| over the bound "
                  "5e-5 + 1.01*2^-8 |ref| + 8 sigma of the weight rounding, which the tests also assert)")
    tr.write_line(f"{'test':70s} {'cases':>5s} {'max|err|':>10s} {'/rms(ref)':>10s} {'/derived':>9s} {'max|lse err|':>12s}")
    for name in sorted(worst):
        w = worst[name]
        tr.write_line(f"{name[:70]:70s} {w['n']:5d} {w['err']:10.2e} {w['rel']:10.2e} {w['tight']:9.2f} {w['lse']:12.2e}")
