import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tiny_inputs():
    """Graph, features and seed batches of the smallest workload, on the host."""
    from paper_2110_08450_amd import synth
    w = synth.WORKLOADS["tiny"]
    return w, synth.make_graph(w), synth.make_features(w), synth.make_seed_batches(w)
