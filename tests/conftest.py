import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def small_problem():
    """N=300 slice of the config-1 recipe with its oracle-built P (perplexity 10, k=30)."""
    import numpy as np
    import oracle
    from paper_1807_11824_amd import synth

    X, _ = synth.config1(n=300, d=50, seed=3)
    P = oracle.build_P(X, 10.0, 30)
    rng = np.random.default_rng(5)
    Y = rng.standard_normal((300, 2)).astype(np.float32) * 3.0
    return dict(X=X, P=P, Y=Y)
