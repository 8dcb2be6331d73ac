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
    from paper_2506_00812_amd.workloads import make_workload
    return make_workload("tiny")


@pytest.fixture(scope="session")
def tiny_oracle(tiny):
    from oracle import OracleIndex
    s = tiny.spec
    return OracleIndex(tiny.vectors, tiny.label_offsets, tiny.label_ids, s.n_labels, s.T, s.graph_degree)
