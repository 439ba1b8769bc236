import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs an MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "slow: takes more than a few seconds on the CPU")


def pytest_sessionfinish(session, exitstatus):
    """The parity comparisons record how much of every bar they used (tests/harness.py); show the worst of each."""
    try:
        import harness
    except ImportError:
        return
    if not harness.STATS:
        return
    worst = harness.dump_stats(os.path.join(ROOT, "gpurun_out", "parity_stats.json"))
    print("\nparity margins (worst over the session):")
    for k in sorted(worst):
        print("  %-32s %.4g   %s" % (k, worst[k][0], worst[k][1]))
