import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X")


@pytest.fixture
def force_route():
    """Force one of the two exact Hamming filters for the duration of a test."""
    import paper_1609_01882_amd as psc
    yield psc.set_filter_route
    psc.set_filter_route("auto")


@pytest.fixture(scope="session")
def tiny_pq():
    """A small trained product quantizer + polysemous renumbering from the oracle, on
    SIFT-like vectors (m=8, 128-D).  Short training: enough for the invariants."""
    import numpy as np
    import oracle as O
    import workloads as W

    xt = W.sift_like(4000, seed=11, stream=W.generators.STREAM_TRAIN)
    cb = O.train_pq(xt, 8, iters=6, seed=3)
    cb_poly, pis, losses = O.optimize_index_assignment(cb, n_iter=60_000, seed=17)
    xb = W.sift_like(5000, seed=11, stream=W.generators.STREAM_DB)
    xq = W.sift_like(12, seed=11, stream=W.generators.STREAM_QUERY)
    codes = O.encode(xb, cb_poly)
    return dict(cb=cb, cb_poly=cb_poly, pis=pis, losses=losses, xb=xb, xq=xq, codes=codes,
                xt=xt, np=np)
