import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import llsa_oracle
    llsa_oracle.build()
    return llsa_oracle


@pytest.fixture(scope="session", autouse=True)
def _parity_stats_file(request):
    """After a session that ran GPU parity comparisons: the observed error figures, for the report."""
    yield
    from tests import harness
    if harness.STATS:
        out = os.path.join(ROOT, "gpurun_out")
        os.makedirs(out, exist_ok=True)
        harness.dump_stats(os.path.join(out, "parity_stats.json"))
