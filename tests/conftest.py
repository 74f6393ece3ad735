import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def cfg1():
    """Configuration 1: Erdos-Renyi n=4096, average degree 8, seed 0, H 4096x16 U[-1,1]."""
    from paper_2504_04673_amd import synth
    g = synth.er_graph(4096, 8, 0)
    H = synth.uniform((4096, 16), 0, synth.STREAM_H)
    return g, H
