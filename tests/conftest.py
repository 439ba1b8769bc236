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
    # DINFER_PARITY_STATS: where to leave the per-test table as JSON (nothing is written without it)
    worst = harness.dump_stats(os.environ.get("DINFER_PARITY_STATS") or None)
    print("\nparity margins (worst over the session):")
    for k in sorted(worst):
        print("  %-32s %.4g   %s" % (k, worst[k][0], worst[k][1]))
