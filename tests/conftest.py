import os
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session", autouse=True)
def _build_oracle():
    from oracle import interp
    interp.build()


_CACHE = {}


@pytest.fixture(scope="session")
def workload_cache():
    """Session cache: (config, j) -> (params, graph, fp64 oracle after forward+backward)."""
    from oracle.interp import Oracle
    from paper_1705_07860_amd import workloads as wl

    def get(name, j=0):
        key = (name, j)
        if key not in _CACHE:
            p, g = wl.make(name, j)
            o = Oracle(g, p, "f64")
            o.forward()
            o.backward(g.root)
            _CACHE[key] = (p, g, o)
        return _CACHE[key]
    return get
