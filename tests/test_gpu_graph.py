"""Parity of the k-NN-graph mode (Section 5) with the oracle (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle as O
import workloads as W
from gpu_util import RTOL, assert_topk_matches

pytestmark = pytest.mark.gpu


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.fixture(scope="module")
def graph_setup():
    import paper_1609_01882_amd as psc
    xt = W.relu_like(4000, seed=90, stream=1)
    idx = psc.Index(256, 8)
    idx.train_pq(xt, iters=5, seed=1)
    idx.optimize_index_assignment(n_iter=30_000, seed=2)
    return psc, idx


@pytest.mark.parametrize("n,ht,k", [(6001, 20, 10), (6001, 64, 10), (40_000, 22, 10), (3000, 26, 100)])
def test_graph_matches_oracle(graph_setup, n, ht, k):
    psc, idx = graph_setup
    x = W.relu_like(n, seed=91, stream=2)
    x_dev = _dev(x)
    codes = idx.encode(x_dev)
    ids, d = idx.knn_graph(x_dev, codes, ht, k)
    torch.cuda.synchronize()
    ids, d, codes_h = ids.cpu().numpy(), d.cpu().numpy(), codes.cpu().numpy()
    assert not np.any(ids == np.arange(n)[:, None])  # never its own neighbour
    rows = np.arange(n) if n <= 6001 else np.unique(np.concatenate(
        [np.arange(40), np.arange(n - 40, n), np.arange(32760, 32776), np.random.default_rng(1).integers(0, n, 200)]))
    lut, _ = idx.build_lut(x_dev[torch.from_numpy(rows).cuda()])
    lut64 = lut.cpu().numpy().astype(np.float64)
    ref = O.scan(lut64, codes_h[rows], codes_h, ht, k, skip_id=rows)
    assert_topk_matches(ids[rows], d[rows], ref, lut64, codes_h[rows], codes_h, ht, what=f"graph n={n} ht={ht}")
    # and the oracle's own graph routine (double-precision tables from the raw vectors)
    sub = rows[:64]
    g = O.knn_graph(x, idx.get_codebook(), codes_h, ht, k, rows=sub)
    fin = np.isfinite(g["dists"])
    assert np.array_equal(fin, np.isfinite(d[sub]))
    assert np.allclose(d[sub][fin], g["dists"][fin], rtol=RTOL)


def test_graph_with_duplicate_vectors(graph_setup):
    """Exact duplicates under another row number stay eligible neighbours (distance of the
    duplicate = the vector's own quantization error), only the row itself is skipped."""
    psc, idx = graph_setup
    x = W.relu_like(500, seed=92, stream=2)
    x = np.concatenate([x, x[:50]])  # rows 500..549 duplicate rows 0..49
    x_dev = _dev(x)
    codes = idx.encode(x_dev)
    ids, d = idx.knn_graph(x_dev, codes, 64, 5)
    torch.cuda.synchronize()
    ids, codes_h = ids.cpu().numpy(), codes.cpu().numpy()
    lut64 = idx.build_lut(x_dev)[0].cpu().numpy().astype(np.float64)
    ref = O.scan(lut64, codes_h, codes_h, 64, 5, skip_id=np.arange(550))
    assert_topk_matches(ids, d.cpu().numpy(), ref, lut64, codes_h, codes_h, 64, what="dups")
    for i in range(50):
        assert (500 + i) in ids[i] and i in ids[500 + i]
