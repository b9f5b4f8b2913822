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
    """With STX_USAGE_REPORT=<file>: how much of its bar every gradient check of the GPU tests used."""
    path = os.environ.get("STX_USAGE_REPORT")
    if not path:
        return
    try:
        from tests import gpu_util as G
    except Exception:
        return
    worst = {}
    for what, used in G.USAGE:
        lo, hi, n = worst.get(what, (used, used, 0))
        worst[what] = (min(lo, used), max(hi, used), n + 1)
    with open(path, "w") as f:
        f.write("check, smallest and largest value over the checks of this run, number of checks\n")
        for what in sorted(worst):
            f.write("%-40s %.4g %.4g %d\n" % (what, *worst[what]))
