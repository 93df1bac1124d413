"""Pins of the oracle's whole search (Section 3.3 two-step strategy; Section 4.2 "dual";
Section 4.1 recall@R)."""
import numpy as np
from scipy.spatial.distance import cdist

import oracle as O
import workloads as W


def _bits(a):
    return np.unpackbits(np.ascontiguousarray(a), axis=1)


def _reference_dual(xq, cb, codes, ht, k):
    """Independent numpy route: full ADC ranking by direct reconstruction, then keep the
    codes whose bitwise distance to the query's code is <= ht, first k."""
    m, _, dsub = cb.shape
    rec = np.concatenate([cb[j][codes[:, j]] for j in range(m)], axis=1)
    d = cdist(xq.astype(np.float64), rec, "sqeuclidean")
    qc = np.stack([cdist(xq[:, j * dsub:(j + 1) * dsub].astype(np.float64), cb[j],
                         "sqeuclidean").argmin(axis=1) for j in range(m)], axis=1).astype(np.uint8)
    h = (_bits(qc)[:, None, :] != _bits(codes)[None, :, :]).sum(axis=2)
    ids = np.full((len(xq), k), -1, dtype=np.int64)
    dist = np.full((len(xq), k), np.inf)
    for q in range(len(xq)):
        order = np.lexsort((np.arange(len(codes)), d[q]))
        keep = order[h[q][order] <= ht][:k]
        ids[q, :len(keep)] = keep
        dist[q, :len(keep)] = d[q][keep]
    return ids, dist, (h <= ht[..., None] if isinstance(ht, np.ndarray) else h <= ht).sum(axis=1)


def test_full_threshold_is_pure_adc(tiny_pq):
    cb, xq, codes = tiny_pq["cb_poly"], tiny_pq["xq"], tiny_pq["codes"][:2000]
    ids, dist, ns = _reference_dual(xq, cb, codes, 64, 25)
    r = O.search_flat(xq, cb, codes, 64, 25)
    assert np.array_equal(r["ids"], ids)
    assert np.allclose(r["dists"], dist, rtol=1e-12)
    assert np.all(r["nsurv"] == len(codes))


def test_dual_is_adc_ranking_restricted_to_survivors(tiny_pq):
    cb, xq, codes = tiny_pq["cb_poly"], tiny_pq["xq"], tiny_pq["codes"][:3000]
    for ht in (8, 16, 22, 28, 36):
        ids, dist, ns = _reference_dual(xq, cb, codes, ht, 40)
        r = O.search_flat(xq, cb, codes, ht, 40)
        assert np.array_equal(r["ids"], ids), ht
        assert np.allclose(r["dists"], dist, rtol=1e-12)
        assert np.array_equal(r["nsurv"], ns)


def test_centroid_database_gives_exact_knn():
    """When every database vector is exactly a concatenation of centroids, ADC distances
    are the true distances, so pure-ADC search == brute-force exact k-NN."""
    rng = np.random.default_rng(8)
    m, dsub = 8, 4
    cb = rng.integers(-20, 21, size=(m, 256, dsub)).astype(np.float64)
    codes = rng.integers(0, 256, size=(700, m)).astype(np.uint8)
    xb = np.concatenate([cb[j][codes[:, j]] for j in range(m)], axis=1)
    xq = rng.integers(-20, 21, size=(9, m * dsub)).astype(np.float64)
    r = O.search_flat(xq, cb, codes, 64, 15)
    gt_ids, gt_d = O.exact_knn(xb, xq, 15)
    assert np.array_equal(r["ids"], gt_ids)
    assert np.array_equal(r["dists"], gt_d)  # integers: exact in floating point
    # exact_knn itself against a library routine
    d = cdist(xq, xb, "sqeuclidean")
    for q in range(len(xq)):
        assert np.array_equal(gt_ids[q], np.lexsort((np.arange(len(xb)), d[q]))[:15])


def test_ties_go_to_lower_id_and_short_lists_are_padded():
    m = 8
    lut = np.zeros((1, m, 256))
    lut[0, 0, :] = np.arange(256)  # distance = first byte
    codes = np.zeros((6, m), np.uint8)
    codes[:, 0] = [5, 3, 5, 3, 9, 3]
    codes[4, 1] = 0xFF  # 8 + popcount(9)=2 -> farther in Hamming from the zero query code
    qc = np.zeros((1, m), np.uint8)
    r = O.scan(lut, qc, codes, 64, 8)
    assert r["ids"][0].tolist() == [1, 3, 5, 0, 2, 4, -1, -1]
    assert r["dists"][0][:6].tolist() == [3, 3, 3, 5, 5, 9]
    assert np.all(np.isinf(r["dists"][0][6:]))
    r = O.scan(lut, qc, codes, 2, 3)  # popcount(5)=2, popcount(3)=2, row 4 has 10 bits
    assert r["ids"][0].tolist() == [1, 3, 5] and r["nsurv"][0] == 5
    r = O.scan(lut, qc, codes, 1, 3)
    assert r["ids"][0].tolist() == [-1, -1, -1] and r["nsurv"][0] == 0
    # external ids and the skipped id of graph mode
    ext = np.array([60, 50, 40, 30, 20, 10])
    r = O.scan(lut, qc, codes, 64, 4, ext_ids=ext, skip_id=np.array([30]))
    assert r["ids"][0].tolist() == [10, 50, 40, 60] and r["nsurv"][0] == 6
    # empty database
    r = O.scan(lut, qc, np.zeros((0, m), np.uint8), 64, 2)
    assert r["ids"][0].tolist() == [-1, -1] and r["nsurv"][0] == 0


def test_recall_at_R():
    ids = np.array([[4, 7, 1], [2, 0, 9], [5, 5, 5]])
    truth = np.array([7, 9, 6])
    assert O.recall_at(ids, truth, 1) == 0.0
    assert abs(O.recall_at(ids, truth, 2) - 1 / 3) < 1e-15
    assert abs(O.recall_at(ids, truth, 3) - 2 / 3) < 1e-15


def test_graph_rows_equal_flat_search_minus_self(tiny_pq):
    """k-NN graph mode (Section 5): row i is the search for x_i, with i itself removed."""
    cb, xb, codes = tiny_pq["cb_poly"], tiny_pq["xb"][:800], tiny_pq["codes"][:800]
    k = 7
    rows = np.array([0, 3, 17, 401, 799])
    g = O.knn_graph(xb, cb, codes, 26, k, rows=rows)
    lut = O.build_lut(xb[rows], cb)
    flat = O.scan(lut, codes[rows], codes, 26, k + 1)
    for t, i in enumerate(rows):
        want = [v for v in flat["ids"][t].tolist() if v != i][:k]
        want += [-1] * (k - len(want))
        assert g["ids"][t].tolist() == want
        assert i in flat["ids"][t]  # the vector finds itself at Hamming distance 0
        assert g["nsurv"][t] == flat["nsurv"][t]


def test_polysemous_filter_beats_plain_numbering():
    """At a comparable filter rate the optimised numbering keeps clearly more of the
    pure-ADC top-10 than the k-means numbering (Section 4.2, Table 1: PQ/dual vs
    PolyD/dual).  Statistical, on a single wide Gaussian (no cluster structure)."""
    kw = dict(seed=31, n_centres=1, sigma=30.0)
    xt = W.sift_like(4000, stream=1, **kw)
    xb = W.sift_like(8000, stream=2, **kw)
    xq = W.sift_like(40, stream=3, **kw)
    cb = O.train_pq(xt, 8, iters=6, seed=3)
    cb_poly, _, _ = O.optimize_index_assignment(cb, n_iter=60_000, seed=17)
    c0, c1 = O.encode(xb, cb), O.encode(xb, cb_poly)
    top = O.search_flat(xq, cb, c0, 64, 10)["ids"]

    def kept(cbk, codes, ht):
        r = O.search_flat(xq, cbk, codes, ht, 10)
        hit = np.mean([len(set(a) & set(b)) / 10 for a, b in zip(r["ids"].tolist(), top.tolist())])
        return hit, r["nsurv"].mean() / len(codes)

    h0, s0 = kept(cb, c0, 24)
    h1, s1 = kept(cb_poly, c1, 24)
    assert s1 < 1.5 * s0          # about the same fraction passes the filter
    assert h1 > 2.0 * h0, (h0, h1, s0, s1)
