import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def orc():
    from oracle import pag_oracle
    pag_oracle.lib()
    return pag_oracle


@pytest.fixture(scope="session")
def cfg1_small():
    """Configuration 1 at reduced size (n = 3000) with brute-force ground truth."""
    import pag_workloads as wl
    w = wl.workload(1, n=3000, nq=200)
    base = wl.make(w, "base")
    q = wl.make(w, "query")
    gt, gtk = wl.brute_force(base, q, w.K, w.metric)
    return w, base, q, gt, gtk


@pytest.fixture(scope="session")
def cfg1_oracle_index(orc, cfg1_small):
    w, base, q, gt, gtk = cfg1_small
    return orc.OracleIndex.build(base, w.metric, deg=w.deg, P=w.P, efC=100, seed=11)
