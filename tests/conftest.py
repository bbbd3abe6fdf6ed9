import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionfinish(session, exitstatus):
    """ASX_PARITY_LOG=<file>: dump the error statistics of every GPU-vs-oracle comparison of the session."""
    path = os.environ.get("ASX_PARITY_LOG")
    if not path:
        return
    import json
    try:
        import parity_util as pu
    except ImportError:
        return
    with open(path, "w") as fh:
        json.dump(pu.STATS_LOG, fh)
