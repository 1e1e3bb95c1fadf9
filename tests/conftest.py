import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "slow: full-size case (minutes)")


def read_golden(name):
    """Parse a tests/golden text fixture: '#' comments, then 'key' lines followed by number rows."""
    out, key = {}, None
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line[0].isalpha():
                key = line
                out[key] = []
            else:
                out[key].append([int(t) for t in line.split()])
    return out


@pytest.fixture(scope="session")
def oracle_mod():
    import oracle
    oracle.build()
    return oracle


def snapshot_from_lists(oracle, X, lists, W):
    """Snapshot whose row u holds `lists[u]` (ids), distances by numpy, all flags new, sorted."""
    n = len(X)
    s = oracle.Snapshot.empty(n, W)
    Xd = X.astype(np.float64)
    for u, ids in enumerate(lists):
        ent = []
        for v in ids:
            dd = float(((Xd[u] - Xd[v]) ** 2).sum())
            if X.dtype == np.float32:
                dd = float(np.float32(dd))
            ent.append((dd, v))
        ent.sort()
        for k, (dd, v) in enumerate(ent):
            s.ids[u, k], s.dist[u, k], s.flags[u, k] = v, dd, 1
        s.deg[u] = len(ent)
    return s


def live(test):
    """Decorator for the cases that run for minutes: their progress lines (Python's and the oracle's own,
    written by C code to stderr) reach the real stdout/stderr even when pytest captures output, so a watcher
    of the run sees that it is alive."""
    import functools

    @functools.wraps(test)
    def wrapper(*args, capfd, **kwargs):
        with capfd.disabled():
            return test(*args, **kwargs)
    import inspect
    sig = inspect.signature(test)
    params = list(sig.parameters.values()) + [inspect.Parameter("capfd", inspect.Parameter.KEYWORD_ONLY)]
    wrapper.__signature__ = sig.replace(parameters=params)
    return wrapper
