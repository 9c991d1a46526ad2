import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def sift10k():
    """Config 1: 10 000 x 128 integer-valued vectors, 1 000 queries (see ggnn_inputs.CONFIGS)."""
    import ggnn_inputs
    return ggnn_inputs.make("sift10k")


@pytest.fixture(scope="session")
def sift10k_oracle_graph(sift10k):
    """The oracle's own build of config 1 (K=24, 3 levels, tau_b=0.5, r=2)."""
    from oracle import ggnn_ref as R
    base, _, cfg = sift10k
    return R.Graph(base, cfg["K"], cfg["levels"]).build()


@pytest.fixture(scope="session")
def sift10k_gt(sift10k):
    from oracle import ggnn_ref as R
    base, queries, cfg = sift10k
    return R.bruteforce(base, queries, cfg["k"])
