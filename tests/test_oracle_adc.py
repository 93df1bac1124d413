"""Pins of the oracle's product-quantizer encoding, ADC tables and ADC distance
(Section 3 opening; Section 4.2 "ADC")."""
import numpy as np
from scipy.spatial.distance import cdist

import oracle as O


def test_lut_matches_library_sqeuclidean(tiny_pq):
    cb, xq = tiny_pq["cb_poly"], tiny_pq["xq"]
    lut = O.build_lut(xq, cb)
    m, _, dsub = cb.shape
    for j in range(m):
        want = cdist(xq[:, j * dsub:(j + 1) * dsub].astype(np.float64), cb[j], "sqeuclidean")
        assert np.allclose(lut[:, j, :], want, rtol=1e-12, atol=1e-9)


def test_encode_is_nearest_centroid(tiny_pq):
    cb, xb, codes = tiny_pq["cb_poly"], tiny_pq["xb"], tiny_pq["codes"]
    m, _, dsub = cb.shape
    for j in range(m):
        d = cdist(xb[:500, j * dsub:(j + 1) * dsub].astype(np.float64), cb[j], "sqeuclidean")
        assert np.array_equal(codes[:500, j], d.argmin(axis=1))


def test_encode_ties_take_lowest_index():
    cb = np.zeros((8, 256, 2))
    cb[:, :, 0] = np.arange(256)[None, :] // 2  # centroids 2c and 2c+1 coincide
    x = np.zeros((3, 16))
    x[1, ::2] = 7.0
    x[2, ::2] = 100.2
    codes = O.encode(x, cb)
    assert np.array_equal(codes[0], np.zeros(8))
    assert np.array_equal(codes[1], np.full(8, 14))
    assert np.array_equal(codes[2], np.full(8, 200))
    qc = O.query_codes(O.build_lut(x, cb))
    assert np.array_equal(qc, codes)


def test_adc_equals_distance_to_reconstruction(tiny_pq):
    """Sum of m table entries == squared distance between the query and the decoded code,
    computed without tables."""
    cb, xq, codes = tiny_pq["cb_poly"], tiny_pq["xq"], tiny_pq["codes"]
    n = len(codes)
    r = O.search_flat(xq, cb, codes, 64, n)  # ht = all bits: every code ranked
    rec = O.decode(codes, cb)
    # reconstruction itself, independently: gather rows of the codebook
    m, _, dsub = cb.shape
    rec2 = np.concatenate([cb[j][codes[:, j]] for j in range(m)], axis=1)
    assert np.array_equal(rec, rec2)
    direct = cdist(xq.astype(np.float64), rec2, "sqeuclidean")
    for q in range(len(xq)):
        assert np.allclose(r["dists"][q], direct[q][r["ids"][q]], rtol=1e-12)
        order = np.lexsort((np.arange(n), direct[q]))
        # ranking identical except where two direct distances tie within rounding
        same = r["ids"][q] == order
        assert same.mean() > 0.999
        assert np.allclose(np.sort(direct[q]), r["dists"][q], rtol=1e-12)


def test_adc_independent_of_index_assignment(tiny_pq):
    """Renumbering centroids changes the bit strings, not the ADC distances (Section 4.2,
    note after the method list): PQ/ADC == PolyD/ADC."""
    cb, cb_poly, pis = tiny_pq["cb"], tiny_pq["cb_poly"], tiny_pq["pis"]
    xb, xq = tiny_pq["xb"][:1500], tiny_pq["xq"]
    c0 = O.encode(xb, cb)
    c1 = O.encode(xb, cb_poly)
    for j in range(8):
        assert np.array_equal(pis[j][c0[:, j]], c1[:, j])  # new index = pi(old index)
        assert np.array_equal(cb_poly[j][pis[j]], cb[j])   # new row pi[i] holds old row i
    r0 = O.search_flat(xq, cb, c0, 64, 50)
    r1 = O.search_flat(xq, cb_poly, c1, 64, 50)
    assert np.array_equal(r0["ids"], r1["ids"])
    assert np.allclose(r0["dists"], r1["dists"], rtol=1e-13)
    # and under an arbitrary random renumbering too
    rng = np.random.default_rng(4)
    cb2 = np.empty_like(cb)
    c2 = np.empty_like(c0)
    for j in range(8):
        p = rng.permutation(256).astype(np.uint8)
        cb2[j] = O.apply_assignment(cb[j], p)
        c2[:, j] = p[c0[:, j]]
    r2 = O.search_flat(xq, cb2, c2, 64, 50)
    assert np.array_equal(r0["ids"], r2["ids"])
