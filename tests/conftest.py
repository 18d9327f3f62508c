import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def o32():
    import oracle
    return oracle.lib("f32")


@pytest.fixture(scope="session")
def o64():
    import oracle
    return oracle.lib("f64")


def pytest_terminal_summary(terminalreporter, exitstatus, config):
    """Parity report of a GPU run: per test function the largest E = max|got - ref| / max(|ref|, tau max|ref|) at the three
    floors tau and the plain inf-norm ratio, printed and written to parity_report.json in the run's output folder."""
    try:
        import gpu_util
    except Exception:
        return
    fam = gpu_util.families()
    if not fam:
        return
    tr = terminalreporter
    tr.write_line("")
    tr.write_line("parity report: E at tau = %s, and |got-ref|_inf / |ref|_inf" % (", ".join("%g" % t for t in gpu_util.REPORT_TAUS)))
    for name in sorted(fam):
        cnt, es, linf = fam[name]
        tr.write_line("  %-86s n=%-5d %s  inf %.2e" % (name, cnt, " ".join("%.2e" % e for e in es), linf))
    out = os.path.join(ROOT, "gpurun_out")
    try:
        os.makedirs(out, exist_ok=True)
        gpu_util.write_report(os.path.join(out, "parity_report.json"))
    except OSError:
        pass
