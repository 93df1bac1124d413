"""Pins of the oracle's index-assignment optimisation (Section 3.1 objective, Section 3.2
annealing).  The trajectory itself depends on the random draws and is unpinned; what is
pinned: the linear map, the loss bookkeeping, the acceptance rule's two limits, the random
generator, and the qualitative effect the paper shows in Figures 1 and 2."""
import os

import numpy as np

import oracle as O
import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _consts():
    out = {}
    for line in open(os.path.join(GOLD, "annealing_constants.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


def _cent(seed=2, dsub=4):
    return np.random.default_rng(seed).normal(size=(256, dsub)) * 10.0


def test_generator_matches_published_vectors():
    for line in open(os.path.join(GOLD, "splitmix64_vectors.txt")):
        line = line.split("#")[0].split()
        if len(line) == 3:
            assert O.draw_u64(int(line[0]), int(line[1])) == int(line[2], 16)


def test_linear_map_matches_binomial_moments():
    """f maps the centroid distances onto the mean d/2 and variance d/4 of the Hamming
    distance between random d-bit strings (Section 3.1)."""
    c = _consts()
    dmat = O.centroid_distances(_cent())
    mu, sigma = O.distance_stats(dmat)
    off = ~np.eye(256, dtype=bool)
    assert np.isclose(mu, dmat[off].mean()) and np.isclose(sigma, dmat[off].std())
    target, weight = O.targets_weights(dmat, mu, sigma, c["alpha"], int(c["nbit"]))
    assert np.isclose(target[off].mean(), c["binomial_mean"])
    assert np.isclose(target[off].var(), c["binomial_var"])
    # closed form, spelled out
    assert np.isclose(O.f_map(mu, mu, sigma), 4.0)
    assert np.isclose(O.f_map(mu + sigma, mu, sigma), 4.0 + np.sqrt(8.0) / 2.0)
    assert np.isclose(O.f_map(mu - 2 * sigma, mu, sigma), 4.0 - np.sqrt(8.0))
    assert np.allclose(weight, 0.5 ** target)
    # Euclidean (not squared) distances between centroids
    cent = _cent()
    assert np.isclose(dmat[3, 200], np.sqrt(((cent[3] - cent[200]) ** 2).sum()))


def test_loss_is_the_weighted_objective():
    dmat = O.centroid_distances(_cent())
    mu, sigma = O.distance_stats(dmat)
    target, weight = O.targets_weights(dmat, mu, sigma)
    pi = np.random.default_rng(1).permutation(256).astype(np.uint8)
    bits = np.unpackbits(pi[:, None], axis=1)
    h = (bits[:, None, :] != bits[None, :, :]).sum(axis=2)
    want = (weight * (h - target) ** 2).sum()
    assert np.isclose(O.polyd_loss(target, weight, pi), want, rtol=1e-12)


def test_swap_delta_equals_full_recomputation():
    dmat = O.centroid_distances(_cent(5))
    mu, sigma = O.distance_stats(dmat)
    target, weight = O.targets_weights(dmat, mu, sigma)
    rng = np.random.default_rng(9)
    pi = rng.permutation(256).astype(np.uint8)
    for _ in range(40):
        a, b = rng.choice(256, size=2, replace=False)
        before = O.polyd_loss(target, weight, pi)
        d = O.swap_delta(target, weight, pi, int(a), int(b))
        pi[a], pi[b] = pi[b], pi[a]
        after = O.polyd_loss(target, weight, pi)
        assert np.isclose(after - before, d, rtol=1e-9, atol=1e-7 * abs(before))


def test_annealing_bookkeeping_and_limits():
    cent = _cent(7)
    c = _consts()
    r = O.anneal(cent, n_iter=20_000, t0=c["t0"], t_decay=c["t_decay_per_500"] ** (1 / 500),
                 alpha=c["alpha"], seed=3, want_trace=True)
    assert sorted(r["pi"].tolist()) == list(range(256))          # still a bijection
    assert np.isclose(r["trace"][0], r["loss_init"])
    assert np.isclose(r["trace"][-1], r["loss_final"], rtol=1e-9)  # running loss == recomputed
    assert r["loss_final"] < 0.8 * r["loss_init"]
    # temperature 0: only improving swaps are accepted -> the loss never rises
    g = O.anneal(cent, n_iter=5_000, t0=0.0, t_decay=1.0, seed=3, want_trace=True)
    assert np.all(np.diff(g["trace"]) <= 1e-9)
    # temperature 1 forever: every proposal is accepted -> pi is the product of all proposed
    # transpositions, which can be replayed from the generator alone
    n = 300
    a = O.anneal(cent, n_iter=n, t0=1.0, t_decay=1.0, seed=12)
    pi = np.arange(256)
    for it in range(n):
        i = O.draw_u64(12, 3 * it) % 256
        j = (i + 1 + O.draw_u64(12, 3 * it + 1) % 255) % 256
        assert i != j
        pi[i], pi[j] = pi[j], pi[i]
    assert np.array_equal(a["pi"], pi)


def test_optimised_numbering_puts_close_centroids_at_small_hamming_distance(tiny_pq):
    """Figure 1: after optimisation, indices differing by one bit belong to close centroids;
    Figure 2: Hamming distance correlates better with true distance."""
    cb, cb_poly, (li, lf) = tiny_pq["cb"], tiny_pq["cb_poly"], tiny_pq["losses"]
    assert np.all(lf < li)
    idx = np.arange(256)
    for j in range(8):
        def one_bit_mean(c):
            return np.mean([np.linalg.norm(c[idx] - c[idx ^ (1 << b)], axis=1).mean() for b in range(8)])
        assert one_bit_mean(cb_poly[j]) < 0.92 * one_bit_mean(cb[j])
    xb = tiny_pq["xb"][:400].astype(np.float64)
    true = ((xb[:, None, :] - xb[None, :, :]) ** 2).sum(axis=2)
    iu = np.triu_indices(400, 1)

    def corr(cbk):
        h = O.hamming_matrix(O.encode(xb, cbk), O.encode(xb, cbk))
        return np.corrcoef(h[iu], np.sqrt(true[iu]))[0, 1]
    assert corr(cb_poly) > corr(cb) + 0.1


def test_kmeans_objective_never_rises():
    x = W.sift_like(3000, seed=2, stream=1)[:, :16]
    cent, obj = O.kmeans(x, 256, 8, seed=1)
    assert np.all(np.diff(obj) <= 1e-6 * obj[0])
    assert cent.shape == (256, 16) and np.isfinite(cent).all()


def test_kmeans_closed_forms():
    """Cases where Lloyd's result is fixed by the mathematics, whatever rows the start draws:
    one centroid is the mean and its objective n times the variance; as many centroids as
    (distinct) points reproduce the points with objective zero; two well separated pairs on a
    line end at the pair means from every possible start."""
    rng = np.random.default_rng(5)
    x = rng.normal(size=(200, 3)) * [1.0, 4.0, 0.5] + [2.0, -1.0, 7.0]
    cent, obj = O.kmeans(x, 1, 3, seed=0)
    assert np.allclose(cent[0], x.mean(axis=0), rtol=0, atol=1e-12)
    assert np.isclose(obj[-1], 200 * x.var(axis=0).sum(), rtol=1e-12)

    pts = rng.permutation(40).astype(np.float64).reshape(20, 2)
    cent, obj = O.kmeans(pts, 20, 2, seed=3)
    assert sorted(map(tuple, cent)) == sorted(map(tuple, pts))
    assert obj[-1] == 0.0

    line = np.array([[0.0], [1.0], [10.0], [11.0]])
    starts = set()
    for seed in range(40):
        starts.add(tuple(sorted(np.random.default_rng(seed).choice(4, size=2, replace=False).tolist())))
        cent, obj = O.kmeans(line, 2, 4, seed=seed)
        assert sorted(cent[:, 0].tolist()) == [0.5, 10.5], seed
        assert obj[-1] == 1.0  # four points at distance 1/2 from their centroid
    assert len(starts) == 6  # every possible pair of starting rows was tried


def test_kmeans_refills_an_empty_cluster():
    """Three copies of one point and one point apart: whenever the start draws two of the copies
    the second centroid attracts nothing (ties go to the lower index) and must be re-seeded with
    the point farthest from the crowded centroid, so every start ends at {0, 5} with objective 0."""
    x = np.array([[0.0, 0.0], [0.0, 0.0], [0.0, 0.0], [5.0, 0.0]])
    seen_refill = False
    for seed in range(12):
        start = x[np.random.default_rng(seed).choice(4, size=2, replace=False)]
        seen_refill |= bool((start == 0).all())
        cent, obj = O.kmeans(x, 2, 3, seed=seed)
        assert sorted(cent[:, 0].tolist()) == [0.0, 5.0] and (cent[:, 1] == 0).all(), seed
        assert obj[-1] == 0.0
    assert seen_refill


def test_kmeans_ends_on_a_fixed_point():
    """After convergence on a small set every centroid is the mean of exactly the points that are
    nearest to it (brute-force distances in numpy, not the oracle's own assignment routine)."""
    x = W.sift_like(300, seed=9, stream=1)[:, :4].astype(np.float64)
    cent, obj = O.kmeans(x, 5, 60, seed=2)
    d = ((x[:, None, :] - cent[None, :, :]) ** 2).sum(axis=2)
    a = d.argmin(axis=1)
    assert obj[-1] == obj[-2]
    for c in range(5):
        assert (a == c).any()
        assert np.allclose(cent[c], x[a == c].mean(axis=0), rtol=0, atol=1e-9)
    assert np.isclose(obj[-1], d.min(axis=1).sum(), rtol=1e-12)


def test_kmeans_from_a_given_start():
    """`start` replaces the seeded draw: one iteration from hand-built centroids has a closed-form
    result (the seed must then play no part), including the order of the returned rows, the
    objective measured at the assignment step, and the refill of a cell the start leaves empty."""
    pts = np.array([[0.0, 0.0], [2.0, 0.0], [0.0, 2.0], [10.0, 10.0], [12.0, 10.0], [20.0, 0.0]])
    start = np.array([[11.0, 9.0], [1.0, 1.0], [21.0, 1.0]])   # cell 0: rows 3,4; cell 1: rows 0,1,2; cell 2: row 5
    for seed in (0, 1, 99):
        cent, obj = O.kmeans(pts, 3, 1, seed=seed, start=start)
        assert np.array_equal(cent, [[11.0, 10.0], [2.0 / 3.0, 2.0 / 3.0], [20.0, 0.0]])
        # squared distances to the *starting* centroids: rows 0-2 -> 2 each, rows 3,4 -> 2 each, row 5 -> 2
        assert obj == [12.0]
    cent, obj = O.kmeans(pts, 3, 2, seed=5, start=start)
    assert np.allclose(obj, [12.0, 2.0 + (4 * 2 / 9 + 2 * (16 / 9 + 4 / 9)) + 0.0], rtol=1e-14)
    assert not np.shares_memory(cent, start) and start[0, 0] == 11.0   # the caller's array is left alone
    # a start that leaves cell 1 empty (ties and nearer rows all go to cell 0): it takes the member
    # of the crowded cell that lies farthest from that cell's centroid, here row 3
    line = np.array([[0.0], [1.0], [2.0], [9.0]])
    cent, obj = O.kmeans(line, 2, 1, seed=0, start=np.array([[1.0], [50.0]]))
    assert obj == [1.0 + 0.0 + 1.0 + 64.0]
    assert cent[:, 0].tolist() == [3.0, 9.0]   # donor mean still counts the row it gives away
