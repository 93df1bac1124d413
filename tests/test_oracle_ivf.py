"""Pins of the oracle's inverted-file search with residual codes (Section 2 "Non-exhaustive
search"; Section 4.3)."""
import numpy as np
from scipy.spatial.distance import cdist

import oracle as O
import workloads as W


def _setup(nlist=12, n=3000, nq=7):
    xt = W.sift_like(3000, seed=41, stream=1)
    xb = W.sift_like(n, seed=41, stream=2)
    xq = W.sift_like(nq, seed=41, stream=3)
    coarse = O.ivf_train_coarse(xt, nlist, iters=5, seed=1)
    res_t = xt - coarse[O.nearest(xt, coarse)[0]]
    cb = O.train_pq(res_t, 8, iters=4, seed=2)
    offsets, codes, ids, list_no = O.ivf_build_lists(xb, coarse, cb)
    return xb, xq, coarse, cb, offsets, codes, ids, list_no


def test_lists_partition_the_database():
    xb, xq, coarse, cb, offsets, codes, ids, list_no = _setup()
    assert offsets[0] == 0 and offsets[-1] == len(xb) and np.all(np.diff(offsets) >= 0)
    assert sorted(ids.tolist()) == list(range(len(xb)))
    d = cdist(xb.astype(np.float64), coarse, "sqeuclidean")
    assert np.array_equal(list_no, d.argmin(axis=1))
    for l in range(len(coarse)):
        members = ids[offsets[l]:offsets[l + 1]]
        assert np.all(list_no[members] == l) and np.all(np.diff(members) > 0)


def test_single_list_with_zero_centroid_is_flat_search():
    xb = W.sift_like(2000, seed=43, stream=2)
    xq = W.sift_like(5, seed=43, stream=3)
    cb = O.train_pq(W.sift_like(2500, seed=43, stream=1), 8, iters=4, seed=2)
    coarse = np.zeros((1, 128))
    offsets, codes, ids, _ = O.ivf_build_lists(xb, coarse, cb)
    assert np.array_equal(ids, np.arange(2000)) and np.array_equal(codes, O.encode(xb, cb))
    for ht in (20, 30, 64):
        a = O.ivf_search(xq, cb, coarse, offsets, codes, ids, 1, ht, 12)
        b = O.search_flat(xq, cb, codes, ht, 12)
        assert np.array_equal(a["ids"], b["ids"]) and np.array_equal(a["dists"], b["dists"])
        assert np.array_equal(a["nsurv"], b["nsurv"])


def test_probing_every_list_without_filter_is_exhaustive_residual_adc():
    xb, xq, coarse, cb, offsets, codes, ids, list_no = _setup()
    nlist = len(coarse)
    r = O.ivf_search(xq, cb, coarse, offsets, codes, ids, nlist, 64, 30)
    # independent route: reconstruct every vector as coarse centroid + decoded residual
    m = 8
    rec = np.empty((len(xb), 128))
    for l in range(nlist):
        sl = slice(offsets[l], offsets[l + 1])
        rec[ids[sl]] = coarse[l] + np.concatenate([cb[j][codes[sl, j]] for j in range(m)], axis=1)
    d = cdist(xq.astype(np.float64), rec, "sqeuclidean")
    for q in range(len(xq)):
        order = np.lexsort((np.arange(len(xb)), d[q]))[:30]
        assert np.allclose(r["dists"][q], d[q][order], rtol=1e-10)
        assert (r["ids"][q] == order).mean() > 0.95  # equal up to rounding-level ties
    assert np.all(r["nsurv"] == len(xb))


def test_probed_lists_are_the_nearest_coarse_centroids_and_filter_is_per_list():
    xb, xq, coarse, cb, offsets, codes, ids, list_no = _setup()
    nprobe, ht, k = 4, 26, 20
    r = O.ivf_search(xq, cb, coarse, offsets, codes, ids, nprobe, ht, k)
    d = cdist(xq.astype(np.float64), coarse, "sqeuclidean")
    for q in range(len(xq)):
        want = np.lexsort((np.arange(len(coarse)), d[q]))[:nprobe]
        assert np.array_equal(r["probed"][q], want)
        # union of per-list flat searches on the residual query, one code per probed list
        cand = []
        ns = 0
        for l in want:
            sl = slice(offsets[l], offsets[l + 1])
            res = (xq[q].astype(np.float64) - coarse[l])[None, :]
            f = O.search_flat(res, cb, codes[sl], ht, k, ext_ids=ids[sl].astype(np.int64))
            ns += f["nsurv"][0]
            cand += [(dd, ii) for dd, ii in zip(f["dists"][0], f["ids"][0]) if ii >= 0]
        cand.sort()
        cand = cand[:k]
        got = [(dd, ii) for dd, ii in zip(r["dists"][q], r["ids"][q]) if ii >= 0]
        assert got == cand
        assert r["nsurv"][q] == ns
    # nprobe larger than the number of lists probes them all
    r2 = O.ivf_search(xq, cb, coarse, offsets, codes, ids, 999, 64, 5)
    assert r2["probed"].shape[1] == len(coarse)


def _union_of_lists(xq_row, cb, coarse, offsets, codes, ids, lists, ht, k, qcodes=None):
    """The definition, one list at a time: flat scan of each given list with the residual query's
    tables (and the given bit string, if any), all candidates ranked together by (distance, id)."""
    cand, ns = [], 0
    for p, l in enumerate(lists):
        sl = slice(offsets[l], offsets[l + 1])
        lut = O.build_lut((xq_row.astype(np.float64) - coarse[l])[None, :], cb)
        qc = O.query_codes(lut) if qcodes is None else qcodes[p][None, :]
        f = O.scan(lut, qc, codes[sl], ht, k, ext_ids=ids[sl].astype(np.int64))
        ns += int(f["nsurv"][0])
        cand += [(dd, ii) for dd, ii in zip(f["dists"][0], f["ids"][0]) if ii >= 0]
    cand.sort()
    return cand[:k], ns


def test_override_with_own_decisions_changes_nothing():
    """Feeding the oracle's own probed lists (and its own per-list bit strings) back in through the
    override arguments must reproduce the unconstrained search bit for bit."""
    xb, xq, coarse, cb, offsets, codes, ids, list_no = _setup()
    nprobe, ht, k = 5, 25, 15
    free = O.ivf_search(xq, cb, coarse, offsets, codes, ids, nprobe, ht, k)
    own_qc = np.empty((len(xq), nprobe, 8), np.uint8)
    for q in range(len(xq)):
        for p, l in enumerate(free["probed"][q]):
            own_qc[q, p] = O.query_codes(O.build_lut((xq[q].astype(np.float64) - coarse[l])[None, :], cb))[0]
    for kw in (dict(probed_in=free["probed"]), dict(qcodes_in=own_qc),
               dict(probed_in=free["probed"], qcodes_in=own_qc)):
        r = O.ivf_search(xq, cb, coarse, offsets, codes, ids, nprobe, ht, k, **kw)
        for key in ("ids", "dists", "nsurv", "probed"):
            assert np.array_equal(r[key], free[key]), (key, list(kw))


def test_overridden_lists_and_bit_strings_are_used_per_query_and_probe():
    """Arbitrary lists per (query, probe) -- not the nearest ones, in no particular order, different
    for every query -- and arbitrary bit strings per (query, probe): the result is the union of the
    per-list scans of exactly those lists under exactly those bit strings.  Catches a wrong stride or
    a transposed index in either override, and a candidate count taken from the unoverridden lists."""
    xb, xq, coarse, cb, offsets, codes, ids, list_no = _setup(nlist=12, n=3000, nq=6)
    rng = np.random.default_rng(77)
    nlist, nprobe, ht, k = len(coarse), 4, 27, 25
    pin = np.stack([rng.permutation(nlist)[:nprobe] for _ in range(len(xq))]).astype(np.int32)
    # make one query probe the longest lists (more candidates than its own nearest lists hold)
    pin[0] = np.argsort(-np.diff(offsets))[:nprobe]
    r = O.ivf_search(xq, cb, coarse, offsets, codes, ids, nprobe, ht, k, probed_in=pin)
    assert np.array_equal(r["probed"], pin)
    for q in range(len(xq)):
        want, ns = _union_of_lists(xq[q], cb, coarse, offsets, codes, ids, pin[q], ht, k)
        got = [(dd, ii) for dd, ii in zip(r["dists"][q], r["ids"][q]) if ii >= 0]
        assert got == want and r["nsurv"][q] == ns, q
    qin = rng.integers(0, 256, size=(len(xq), nprobe, 8)).astype(np.uint8)
    r = O.ivf_search(xq, cb, coarse, offsets, codes, ids, nprobe, 30, k, probed_in=pin, qcodes_in=qin)
    seen = 0
    for q in range(len(xq)):
        want, ns = _union_of_lists(xq[q], cb, coarse, offsets, codes, ids, pin[q], 30, k, qcodes=qin[q])
        got = [(dd, ii) for dd, ii in zip(r["dists"][q], r["ids"][q]) if ii >= 0]
        assert got == want and r["nsurv"][q] == ns, q
        seen += ns
    assert seen > 0  # random 64-bit strings at threshold 30 do let some codes through


def test_overrides_with_more_probes_than_lists():
    """nprobe above the number of lists is clipped; the override arrays then have nlist columns."""
    xb, xq, coarse, cb, offsets, codes, ids, list_no = _setup(nlist=5, n=1500, nq=3)
    nlist = len(coarse)
    pin = np.stack([np.roll(np.arange(nlist), q + 1) for q in range(len(xq))]).astype(np.int32)
    qin = np.random.default_rng(3).integers(0, 256, size=(len(xq), nlist, 8)).astype(np.uint8)
    r = O.ivf_search(xq, cb, coarse, offsets, codes, ids, 50, 31, 40, probed_in=pin, qcodes_in=qin)
    assert r["probed"].shape == (len(xq), nlist) and np.array_equal(r["probed"], pin)
    for q in range(len(xq)):
        want, ns = _union_of_lists(xq[q], cb, coarse, offsets, codes, ids, pin[q], 31, 40, qcodes=qin[q])
        got = [(dd, ii) for dd, ii in zip(r["dists"][q], r["ids"][q]) if ii >= 0]
        assert got == want and r["nsurv"][q] == ns
    # every list probed, no filter: the order of the lists cannot matter
    a = O.ivf_search(xq, cb, coarse, offsets, codes, ids, 50, 64, 40, probed_in=pin)
    b = O.ivf_search(xq, cb, coarse, offsets, codes, ids, 50, 64, 40)
    assert np.array_equal(a["ids"], b["ids"]) and np.array_equal(a["dists"], b["dists"])
