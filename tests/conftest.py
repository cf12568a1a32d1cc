import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tiny():
    """Tiny config on the CPU: graph, all training vertices, the partition's training vertices."""
    from workloads import synth as S
    g = S.make_graph(S.TINY, "cpu")
    T = S.make_training_set(S.TINY, "cpu")
    Tk = S.local_training_set(S.TINY, T)
    return S.TINY, g, T, Tk
