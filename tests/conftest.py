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
    """A clustered problem a few tiles wide with a ragged tail, shared by the CPU pins."""
    import dataclasses

    import numpy as np

    import oracle
    import workloads as W

    w = dataclasses.replace(W.CONFIGS[1], N=3001, K=37, T=20)
    cw = W.codewords(w)
    codes = W.codes_numpy(w)
    centers = codes[W.init_center_indices(w)].copy()
    tables = oracle.build_tables(cw)
    return dict(w=w, cw=cw, codes=codes, centers=centers, tables=tables, np=np)
