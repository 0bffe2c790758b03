import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as _oracle
    _oracle.lib()
    return _oracle


def pytest_terminal_summary(terminalreporter):
    """The margin of every scalar-gradient check of the session: error over the stated tolerance."""
    try:
        import gpu_util
    except Exception:
        return
    if not gpu_util.SCALAR_LOG:
        return
    tr = terminalreporter
    tr.write_sep("-", "scalar gradients: |gpu - oracle| / (1e-6 + 1e-5 |oracle|)")
    strict = [r for r in gpu_util.SCALAR_LOG if r[3] == "strict"]
    other = [r for r in gpu_util.SCALAR_LOG if r[3] != "strict"]
    worst = sorted(strict, key=lambda r: -r[2])[:12]
    tr.write_line("%d checks within the stated tolerance; the largest ratios:" % len(strict))
    for label, name, ratio, _ in worst:
        tr.write_line("  %-60s %-8s %.3g" % (label, name, ratio))
    tr.write_line("%d checks of sums that cancel (|oracle| < 1e-3 of the size of what is added up), judged by 2e-7 of that size:" % len(other))
    for label, name, ratio, how in other:
        tr.write_line("  %-60s %-8s %.3g  %s" % (label, name, ratio, how))
