"""Pins of the oracle's ranking loss (Section 3.1 "Ranking loss"), of its annealing (Section 3.2)
and of the alternative filter that counts differing indexes (Section 3.3; "disidx" in Section 4.2)."""
import numpy as np

import oracle as O
import workloads as W


def _cent(seed, dsub=6):
    return np.random.default_rng(seed).normal(size=(256, dsub))


def _hd(pi):
    bits = np.unpackbits(np.asarray(pi, np.uint8)[:, None], axis=1)
    return (bits[:, None, :] != bits[None, :, :]).sum(axis=2)


def _loss_numpy(dmat, pi):
    """The objective straight from its definition with numpy broadcasting: for every ordered pair
    (i, j), j != i: weight 1 / rank(i, j), rank = number of centroids strictly nearer to i than j
    (i itself is one), times the harmonic number of the count of k with d_ij < d_ik and
    h(pi_i, pi_j) > h(pi_i, pi_k)."""
    h = _hd(pi)
    harmonic = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, 257))])
    total = 0.0
    for i in range(256):
        viol = ((dmat[i][:, None] < dmat[i][None, :]) & (h[i][:, None] > h[i][None, :])).sum(axis=1)   # [j]
        rank = (dmat[i][None, :] < dmat[i][:, None]).sum(axis=1)
        for j in range(256):
            if j != i and rank[j] > 0:
                total += harmonic[viol[j]] / rank[j]
    return total


def test_harmonic_sums():
    assert [O.ell(r) for r in (0, 1, 2, 4)] == [0.0, 1.0, 1.5, 1.0 + 0.5 + 1.0 / 3.0 + 0.25]


def test_ranks_are_places_in_the_sorted_neighbour_list():
    dmat = O.centroid_distances(_cent(1))
    rank = O.neighbour_ranks(dmat)
    assert np.all(np.diag(rank) == 0)
    for i in (0, 17, 255):
        order = np.argsort(dmat[i], kind="stable")           # i itself first (distance 0)
        assert order[0] == i
        assert np.array_equal(rank[i][order], np.arange(256))  # distinct distances: place = rank
    # duplicates of a centroid share its rank
    c = _cent(2)
    c[9] = c[4]
    rank = O.neighbour_ranks(O.centroid_distances(c))
    assert rank[4, 9] == 0 and rank[9, 4] == 0 and rank[30, 4] == rank[30, 9]


def test_loss_equals_its_definition():
    rng = np.random.default_rng(3)
    dmat = O.centroid_distances(_cent(3))
    rank = O.neighbour_ranks(dmat)
    for pi in (np.arange(256), rng.permutation(256)):
        pi = pi.astype(np.uint8)
        assert np.isclose(O.polyr_loss(dmat, rank, pi), _loss_numpy(dmat, pi), rtol=1e-12)
    # single counts, by hand: k violates the pair (i, j) iff it is farther than j yet nearer in bits
    pi = rng.permutation(256).astype(np.uint8)
    h = _hd(pi)
    for i, j in ((0, 1), (200, 13), (77, 78)):
        want = sum(1 for k in range(256) if dmat[i, j] < dmat[i, k] and h[i, j] > h[i, k])
        assert O.rank_violations(dmat, pi, i, j) == want


def test_hypercube_codebook_is_ranked_perfectly_by_its_own_bits():
    """Centroids at the 256 vertices of the cube {0,1}^8, numbered by their own coordinates: the
    squared distance between two centroids IS the Hamming distance between their indices, so no
    pair is ever ranked wrongly and the loss is exactly zero; any transposition spoils that."""
    cent = np.unpackbits(np.arange(256, dtype=np.uint8)[:, None], axis=1).astype(np.float64)
    dmat = O.centroid_distances(cent)
    rank = O.neighbour_ranks(dmat)
    pi = np.arange(256, dtype=np.uint8)
    assert O.polyr_loss(dmat, rank, pi) == 0.0
    pj = pi.copy()
    pj[1], pj[254] = pj[254], pj[1]
    assert O.polyr_loss(dmat, rank, pj) > 0.0
    assert O.polyr_swap_delta(dmat, rank, pi, 1, 254) == O.polyr_loss(dmat, rank, pj)
    # a bit-flip relabelling (xor with a constant) keeps every Hamming distance: still zero
    assert O.polyr_loss(dmat, rank, pi ^ np.uint8(0x5A)) == 0.0


def test_swap_delta_equals_full_recomputation():
    rng = np.random.default_rng(4)
    dmat = O.centroid_distances(_cent(4))
    rank = O.neighbour_ranks(dmat)
    pi = rng.permutation(256).astype(np.uint8)
    base = O.polyr_loss(dmat, rank, pi)
    for a, b in ((0, 255), (3, 4), (100, 17), (64, 192)):
        pj = pi.copy()
        pj[a], pj[b] = pj[b], pj[a]
        assert np.isclose(O.polyr_swap_delta(dmat, rank, pi, a, b), O.polyr_loss(dmat, rank, pj) - base,
                          rtol=0, atol=1e-9)
    assert O.polyr_swap_delta(dmat, rank, pi, 5, 9) == O.polyr_swap_delta(dmat, rank, pi, 9, 5)


def test_annealing_on_the_ranking_loss():
    cent = _cent(5)
    r = O.anneal_ranking(cent, n_iter=250, t0=0.0, seed=8, want_trace=True)    # temperature 0: greedy
    assert sorted(r["pi"].tolist()) == list(range(256))
    assert np.all(np.diff(r["trace"]) <= 1e-9)                                  # never accepts a worse state
    assert r["loss_final"] < r["loss_init"]
    dmat = O.centroid_distances(cent)
    assert np.isclose(r["loss_final"], O.polyr_loss(dmat, O.neighbour_ranks(dmat), r["pi"]), rtol=1e-12)
    assert np.isclose(r["trace"][-1], r["loss_final"], rtol=1e-9)               # tracked changes add up
    # same proposals as the annealing on the distance loss: with every proposal accepted (t = 1) both
    # walks end on the same permutation
    a = O.anneal_ranking(cent, n_iter=40, t0=1.0, t_decay=1.0, seed=3)
    b = O.anneal(cent, n_iter=40, t0=1.0, t_decay=1.0, seed=3)
    assert np.array_equal(a["pi"], b["pi"])


def test_counting_differing_indexes():
    a = np.array([1, 2, 3, 4, 5, 6, 7, 8], np.uint8)
    assert O.disidx(a, a) == 0
    assert O.disidx(a, a ^ np.uint8(0xFF)) == 8
    b = a.copy()
    b[2] ^= 1          # one index differs by a single bit, another by all eight: two differing indexes
    b[6] ^= 0xFF
    assert O.disidx(a, b) == 2 and O.hamming(a, b) == 9
    assert O.disidx(np.zeros(16, np.uint8), np.eye(16, dtype=np.uint8)[3] * 200) == 1


def test_disidx_scan_is_the_adc_ranking_restricted_to_its_survivors(tiny_pq):
    cb, xq, codes = tiny_pq["cb_poly"], tiny_pq["xq"], tiny_pq["codes"][:3000]
    lut = O.build_lut(xq, cb)
    qc = O.query_codes(lut)
    full = O.scan(lut, qc, codes, 64, len(codes))
    ndiff = (qc[:, None, :] != codes[None, :, :]).sum(axis=2)
    for t in (0, 3, 5, 7, 8):
        r = O.scan(lut, qc, codes, t, 30, filter="disidx")
        assert np.array_equal(r["nsurv"], (ndiff <= t).sum(axis=1))
        for q in range(len(xq)):
            keep = [i for i in full["ids"][q] if ndiff[q, i] <= t][:30]
            assert r["ids"][q][:len(keep)].tolist() == keep and np.all(r["ids"][q][len(keep):] == -1)
    assert np.array_equal(O.scan(lut, qc, codes, 8, 30, filter="disidx")["ids"], O.scan(lut, qc, codes, 64, 30)["ids"])


def test_ranking_by_code_distance_alone():
    """The "binary" and "disidx" comparison methods: the database ordered by (code distance, id)."""
    codes = np.array([[0, 0, 0, 0, 0, 0, 0, 0], [1, 0, 0, 0, 0, 0, 0, 0], [255, 0, 0, 0, 0, 0, 0, 0],
                      [1, 1, 0, 0, 0, 0, 0, 0], [0, 0, 0, 0, 0, 0, 0, 0], [3, 3, 3, 0, 0, 0, 0, 0]], np.uint8)
    q = np.zeros((1, 8), np.uint8)
    ids, d = O.search_by_code_distance(q, codes, 8, "hamming")
    assert ids[0].tolist() == [0, 4, 1, 3, 5, 2, -1, -1] and d[0][:6].tolist() == [0, 0, 1, 2, 6, 8]
    ids, d = O.search_by_code_distance(q, codes, 6, "disidx")
    assert ids[0].tolist() == [0, 4, 1, 2, 3, 5] and d[0].tolist() == [0, 0, 1, 1, 2, 3]
    # against the filter: the first nsurv(t) entries of the ranking are exactly the filter's survivors
    rng = np.random.default_rng(9)
    codes = W.random_codes(500, 8, seed=2)
    qc = codes[rng.integers(0, 500, size=4)] ^ rng.integers(0, 4, size=(4, 8)).astype(np.uint8)
    lut = np.zeros((4, 8, 256))
    ids, d = O.search_by_code_distance(qc, codes, 500, "hamming")
    for t in (10, 25, 30):
        s = O.scan(lut, qc, codes, t, 500, want_bitmap=True)
        for q_ in range(4):
            ns = int(s["nsurv"][q_])
            assert sorted(ids[q_][:ns].tolist()) == np.flatnonzero(s["bitmap"][q_]).tolist()
            assert ns == 500 or d[q_][ns] > t
