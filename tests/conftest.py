import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


MARGIN = 1e-3  # every tested distance stays at least this far from tau


def oracle_arrays(grads):
    from paper_2412_18052_amd import workloads as wl
    return [wl.to_host_array(g) for g in grads]


def workload_with_margin(name, P=None, N=None, seed=0, device="cpu", max_tries=16):
    """Draw a workload whose oracle distances all keep MARGIN from tau.

    The seed is bumped until that holds. Returns (workload, grads, oracle
    result tuple (out, mask, dist, count))."""
    from oracle import gaf_oracle
    from paper_2412_18052_amd import workloads as wl
    for k in range(max_tries):
        w, grads = wl.generate(name, seed + k, P=P, N=N, device=device)
        res = gaf_oracle.aggregate(oracle_arrays(grads), np.float32(w.tau))
        if np.all(np.abs(res[2][1:] - float(np.float32(w.tau))) >= MARGIN):
            return w, grads, res
    raise RuntimeError("no seed in %d tries keeps the margin for %s" % (max_tries, name))


@pytest.fixture(scope="session")
def oracle():
    from oracle import gaf_oracle
    gaf_oracle.build()
    return gaf_oracle
