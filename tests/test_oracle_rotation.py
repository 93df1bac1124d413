"""Pins of the oracle's transformation in front of the product quantizer (Section 4.3: rotation
before encoding; additional results: dimension reduction inside the same transformation)."""
import numpy as np
from scipy.spatial.distance import cdist

import oracle as O
import workloads as W


def _orthogonal(d, seed):
    q, r = np.linalg.qr(np.random.default_rng(seed).standard_normal((d, d)))
    return q * np.sign(np.diag(r))


def test_hand_computed_products():
    r = np.array([[1.0, 2.0, 3.0], [0.0, -1.0, 4.0]])          # 3-D -> 2-D
    x = np.array([[1.0, 1.0, 1.0], [2.0, 0.0, -1.0], [0.0, 5.0, 0.5]])
    assert np.array_equal(O.rotate(x, r), [[6.0, 3.0], [-1.0, -4.0], [11.5, -3.0]])
    assert np.array_equal(O.rotate(x, np.eye(3)), x)
    perm = np.eye(3)[[2, 0, 1]]                                  # output coordinate c = input coordinate perm[c]
    assert np.array_equal(O.rotate(x, perm), x[:, [2, 0, 1]])
    assert np.array_equal(O.rotate(x, np.eye(3)[:2]), x[:, :2])  # keeping the first two coordinates


def test_composition_and_linearity():
    rng = np.random.default_rng(3)
    x, z = rng.standard_normal((50, 24)), rng.standard_normal((50, 24))
    r1, r2 = rng.standard_normal((16, 24)), rng.standard_normal((8, 16))
    assert np.allclose(O.rotate(O.rotate(x, r1), r2), O.rotate(x, r2 @ r1), rtol=1e-12, atol=1e-12)
    assert np.allclose(O.rotate(2.0 * x - z, r1), 2.0 * O.rotate(x, r1) - O.rotate(z, r1), rtol=1e-12, atol=1e-12)


def test_a_rotation_changes_neither_distances_nor_exact_neighbours():
    rng = np.random.default_rng(6)   # (a little noise: the integer-valued vectors have exactly tied distances)
    x = W.sift_like(600, seed=5, stream=2).astype(np.float64) + rng.random((600, 128))
    q = W.sift_like(9, seed=5, stream=3).astype(np.float64) + rng.random((9, 128))
    r = _orthogonal(128, 1)
    xr, qr = O.rotate(x, r), O.rotate(q, r)
    assert np.allclose(cdist(qr, xr, "sqeuclidean"), cdist(q, x, "sqeuclidean"), rtol=1e-10)
    a, b = O.exact_knn(x, q, 10), O.exact_knn(xr, qr, 10)
    assert np.array_equal(a[0], b[0]) and np.allclose(a[1], b[1], rtol=1e-10)


def test_rotation_inside_the_sub_spaces_leaves_codes_and_adc_unchanged(tiny_pq):
    """A block-diagonal orthogonal matrix (one rotation per sub-space) applied to vectors and
    centroids alike maps the product quantizer onto itself: same codes, same table entries, same
    search result -- the ADC side of the codes does not see it."""
    cb, xb, xq = tiny_pq["cb_poly"], tiny_pq["xb"][:1500], tiny_pq["xq"]
    m, _, dsub = cb.shape
    r = np.zeros((m * dsub, m * dsub))
    cb_r = np.empty_like(cb)
    for j in range(m):
        blk = _orthogonal(dsub, 10 + j)
        r[j * dsub:(j + 1) * dsub, j * dsub:(j + 1) * dsub] = blk
        cb_r[j] = cb[j] @ blk.T
    codes = O.encode(xb, cb)
    codes_r = O.encode(O.rotate(xb, r), cb_r)
    assert (codes != codes_r).mean() < 1e-3                       # near-ties only
    lut, lut_r = O.build_lut(xq, cb), O.build_lut(O.rotate(xq, r), cb_r)
    assert np.allclose(lut, lut_r, rtol=1e-9, atol=1e-6)
    a = O.scan(lut, O.query_codes(lut), codes, 26, 20)
    b = O.scan(lut_r, O.query_codes(lut), codes, 26, 20)
    assert np.array_equal(a["ids"], b["ids"]) and np.allclose(a["dists"], b["dists"], rtol=1e-9)


def test_projection_onto_leading_directions_keeps_what_they_hold():
    """Dimension reduction inside the transformation: for vectors that live in a 40-dimensional
    subspace of 128-D, projecting onto an orthonormal basis of that subspace (a 40 x 128 matrix)
    keeps every pairwise distance."""
    rng = np.random.default_rng(12)
    basis = _orthogonal(128, 4)[:40]                              # 40 orthonormal rows
    x = rng.standard_normal((300, 40)) @ basis
    y = O.rotate(x, basis)
    assert y.shape == (300, 40)
    assert np.allclose(cdist(y, y, "sqeuclidean"), cdist(x, x, "sqeuclidean"), rtol=1e-9, atol=1e-9)
