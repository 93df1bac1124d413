"""Pins of the oracle's inverted multi-index search (Section 2 "Non-exhaustive search"; Section 4.3;
caption of Table 2: caps on visited lists and on distance evaluations)."""
import numpy as np
from scipy.spatial.distance import cdist

import oracle as O
import workloads as W


def _setup(k1=6, k2=5, n=3000, nq=6, seed=51):
    xt = W.sift_like(3000, seed=seed, stream=1)
    xb = W.sift_like(n, seed=seed, stream=2)
    xq = W.sift_like(nq, seed=seed, stream=3)
    c1, c2 = O.imi_train_coarse(xt, k1, k2, iters=5, seed=1)
    cell_t = O.nearest(xt[:, :64], c1)[0] * k2 + O.nearest(xt[:, 64:], c2)[0]
    res_t = xt - np.concatenate([c1[cell_t // k2], c2[cell_t % k2]], axis=1)
    cb = O.train_pq(res_t, 8, iters=4, seed=2)
    offsets, codes, ids, cell = O.imi_build_lists(xb, c1, c2, cb)
    return xb, xq, c1, c2, cb, offsets, codes, ids, cell


def _cell_centroids(c1, c2):
    return np.concatenate([np.repeat(c1, len(c2), axis=0), np.tile(c2, (len(c1), 1))], axis=1)   # row a*K2+b


def test_cells_partition_the_database():
    xb, xq, c1, c2, cb, offsets, codes, ids, cell = _setup()
    cc = _cell_centroids(c1, c2)
    assert offsets[0] == 0 and offsets[-1] == len(xb) and len(offsets) == 31
    assert sorted(ids.tolist()) == list(range(len(xb)))
    # nearest half-centroids = nearest cell centroid (the squared distance splits over the halves)
    assert np.array_equal(cell, cdist(xb.astype(np.float64), cc, "sqeuclidean").argmin(axis=1))
    for l in range(30):
        members = ids[offsets[l]:offsets[l + 1]]
        assert np.all(cell[members] == l) and np.all(np.diff(members) > 0)


def test_cells_are_visited_in_order_of_distance_to_the_cell_centroid():
    xb, xq, c1, c2, cb, offsets, codes, ids, cell = _setup()
    d = cdist(xq.astype(np.float64), _cell_centroids(c1, c2), "sqeuclidean")
    r = O.imi_search(xq, cb, c1, c2, offsets, codes, ids, 30, 0, 64, 5)
    for q in range(len(xq)):
        want = np.lexsort((np.arange(30), d[q]))
        assert np.array_equal(r["cells"][q], want)
        assert np.all(np.diff(d[q][r["cells"][q]]) >= 0)
        a, b = divmod(int(r["cells"][q, 0]), 5)
        assert a == cdist(xq[q:q + 1, :64], c1).argmin() and b == cdist(xq[q:q + 1, 64:], c2).argmin()
    assert np.all(r["ncodes"] == len(xb)) and np.all(r["nsurv"] == len(xb))


def test_all_cells_without_filter_is_exhaustive_residual_adc():
    xb, xq, c1, c2, cb, offsets, codes, ids, cell = _setup()
    r = O.imi_search(xq, cb, c1, c2, offsets, codes, ids, 30, 0, 64, 25)
    cc = _cell_centroids(c1, c2)
    rec = np.empty((len(xb), 128))
    for l in range(30):
        sl = slice(offsets[l], offsets[l + 1])
        rec[ids[sl]] = cc[l] + np.concatenate([cb[j][codes[sl, j]] for j in range(8)], axis=1)
    d = cdist(xq.astype(np.float64), rec, "sqeuclidean")
    for q in range(len(xq)):
        order = np.lexsort((np.arange(len(xb)), d[q]))[:25]
        assert np.allclose(r["dists"][q], d[q][order], rtol=1e-10)
        assert (r["ids"][q] == order).mean() > 0.9


def test_caps_on_cells_and_on_codes():
    xb, xq, c1, c2, cb, offsets, codes, ids, cell = _setup()
    sizes = np.diff(offsets)
    full = O.imi_search(xq, cb, c1, c2, offsets, codes, ids, 30, 0, 26, 10)["cells"]
    for max_lists, max_codes in ((4, 0), (30, 700), (3, 100000), (7, 250), (1, 1), (30, 1)):
        r = O.imi_search(xq, cb, c1, c2, offsets, codes, ids, max_lists, max_codes, 26, 10)
        for q in range(len(xq)):
            taken = r["cells"][q][r["cells"][q] >= 0]
            assert np.array_equal(taken, full[q][:len(taken)])              # a prefix of the full order
            assert np.all(r["cells"][q][len(taken):] == -1)
            run = np.cumsum(sizes[taken])
            assert r["ncodes"][q] == (run[-1] if len(run) else 0)
            # stops at the first of: max_lists cells taken, or the codes held reach max_codes
            hit_codes = max_codes > 0 and run[-1] >= max_codes
            assert len(taken) == max_lists or hit_codes or len(taken) == 30
            if max_codes > 0 and len(taken) > 1:
                assert run[-2] < max_codes                                    # the cap was not reached a cell earlier
            assert len(taken) <= max_lists
            # the result is the union of per-cell flat searches on the residual query
            cand = []
            for l in taken:
                sl = slice(offsets[l], offsets[l + 1])
                res = (xq[q].astype(np.float64) - np.concatenate([c1[l // 5], c2[l % 5]]))[None, :]
                f = O.search_flat(res, cb, codes[sl], 26, 10, ext_ids=ids[sl].astype(np.int64))
                cand += [(dd, ii) for dd, ii in zip(f["dists"][0], f["ids"][0]) if ii >= 0]
            cand.sort()
            got = [(dd, ii) for dd, ii in zip(r["dists"][q], r["ids"][q]) if ii >= 0]
            assert got == cand[:10]


def test_a_second_quantizer_with_one_centroid_is_the_plain_inverted_file():
    """K2 = 1: the cells are the lists of an inverted file whose coarse centroids are the first-half
    centroids completed by the one second-half centroid; the order of cells is the order of lists."""
    xt = W.sift_like(2500, seed=52, stream=1)
    xb = W.sift_like(2500, seed=52, stream=2)
    xq = W.sift_like(5, seed=52, stream=3)
    c1, c2 = O.imi_train_coarse(xt, 9, 1, iters=4, seed=3)
    coarse = np.concatenate([c1, np.repeat(c2, 9, axis=0)], axis=1)
    cb = O.train_pq(xt - coarse[O.nearest(xt, coarse)[0]], 8, iters=3, seed=2)
    o1, cd1, id1, _ = O.imi_build_lists(xb, c1, c2, cb)
    o2, cd2, id2, _ = O.ivf_build_lists(xb, coarse, cb)
    assert np.array_equal(o1, o2) and np.array_equal(cd1, cd2) and np.array_equal(id1, id2)
    for nprobe, ht in ((3, 24), (9, 64), (1, 30)):
        a = O.imi_search(xq, cb, c1, c2, o1, cd1, id1, nprobe, 0, ht, 12)
        b = O.ivf_search(xq, cb, coarse, o2, cd2, id2, nprobe, ht, 12)
        assert np.array_equal(a["cells"], b["probed"])
        assert np.array_equal(a["ids"], b["ids"]) and np.allclose(a["dists"], b["dists"], rtol=1e-12)
        assert np.array_equal(a["nsurv"], b["nsurv"])


def test_overridden_cells_and_bit_strings():
    xb, xq, c1, c2, cb, offsets, codes, ids, cell = _setup()
    free = O.imi_search(xq, cb, c1, c2, offsets, codes, ids, 6, 500, 25, 15)
    again = O.imi_search(xq, cb, c1, c2, offsets, codes, ids, 6, 500, 25, 15, cells_in=free["cells"])
    for key in ("ids", "dists", "nsurv", "cells", "ncodes"):
        assert np.array_equal(free[key], again[key]), key
    rng = np.random.default_rng(5)
    cin = np.full((len(xq), 4), -1, np.int32)
    for q in range(len(xq)):
        nc = 1 + q % 4
        cin[q, :nc] = rng.permutation(30)[:nc]
    qin = rng.integers(0, 256, size=(len(xq), 4, 8)).astype(np.uint8)
    r = O.imi_search(xq, cb, c1, c2, offsets, codes, ids, 4, 0, 31, 20, cells_in=cin, qcodes_in=qin)
    assert np.array_equal(r["cells"], cin)
    for q in range(len(xq)):
        cand, ns = [], 0
        for p, l in enumerate(cin[q][cin[q] >= 0]):
            sl = slice(offsets[l], offsets[l + 1])
            lut = O.build_lut((xq[q].astype(np.float64) - np.concatenate([c1[l // 5], c2[l % 5]]))[None, :], cb)
            f = O.scan(lut, qin[q, p][None, :], codes[sl], 31, 20, ext_ids=ids[sl].astype(np.int64))
            ns += int(f["nsurv"][0])
            cand += [(dd, ii) for dd, ii in zip(f["dists"][0], f["ids"][0]) if ii >= 0]
        cand.sort()
        assert [(dd, ii) for dd, ii in zip(r["dists"][q], r["ids"][q]) if ii >= 0] == cand[:20]
        assert r["nsurv"][q] == ns
