"""CPU-side checks of the HIP library: it loads, exports every symbol the header declares,
rejects bad arguments, and its host-side training obeys the same invariants as the oracle's.
No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle as O
import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def psc():
    import paper_1609_01882_amd as p
    if not os.path.exists(p.lib_path()):
        import __graft_entry__ as g
        g.build()
    return p


def _declared():
    text = open(os.path.join(ROOT, "include", "psc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(psc_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(psc):
    lib = C.CDLL(psc.lib_path())
    names = _declared()
    assert len(names) >= 16
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(psc.exported_symbols()) == names
    assert psc.version() >= 100


def test_binding_constants_match_the_header(psc):
    from paper_1609_01882_amd import binding
    text = open(os.path.join(ROOT, "include", "psc.h")).read()
    defs = {k: int(v.strip("()")) for k, v in re.findall(r"^#define (PSC_[A-Z_]+) (\(?-?\d+\)?)$", text, flags=re.M)}
    assert {k: defs[f"PSC_ROUTE_{k.upper()}"] for k in binding.ROUTES} == binding.ROUTES
    assert defs["PSC_MAX_K"] == binding.PSC_MAX_K == psc.PSC_MAX_K
    assert (defs["PSC_START_SEEDED"], defs["PSC_START_CURRENT"]) == (binding.PSC_START_SEEDED, binding.PSC_START_CURRENT)
    assert defs["PSC_OK"] == 0 and all(defs[e] < 0 for e in ("PSC_EINVAL", "PSC_ESTATE", "PSC_EHIP", "PSC_ENOMEM"))


def test_argument_errors(psc):
    with pytest.raises(psc.PscError):
        psc.Index(128, 7)
    with pytest.raises(psc.PscError):
        psc.Index(130, 8)
    idx = psc.Index(128, 8)
    with pytest.raises(psc.PscError):
        idx.get_codebook()  # nothing trained yet
    with pytest.raises(psc.PscError):
        idx.train_pq(np.zeros((10, 128), np.float32))  # too few vectors
    assert psc.scan_workspace_bytes(8, 100, 1000, 10) > 0
    assert psc.scan_workspace_bytes(12, 100, 1000, 10) == 0
    assert psc.scan_workspace_bytes(8, 100, 1000, 0) == 0
    assert psc.scan_workspace_bytes(8, 100, 1000, psc.PSC_MAX_K + 1) == 0


def test_codebook_round_trip(psc):
    idx = psc.Index(64, 16)
    cb = np.random.default_rng(0).normal(size=(16, 256, 4)).astype(np.float32)
    idx.set_codebook(cb)
    assert np.array_equal(idx.get_codebook(), cb)


def test_host_kmeans_quality(psc):
    """The library's k-means must quantize about as well as the oracle's (different seeds and
    start, so only the quantization error is compared)."""
    xt = W.sift_like(4000, seed=11, stream=1)
    idx = psc.Index(128, 8)
    idx.train_pq(xt, iters=6, seed=3)
    cb = idx.get_codebook().astype(np.float64)
    cb_ref = O.train_pq(xt, 8, iters=6, seed=3)
    xe = W.sift_like(2000, seed=11, stream=2)

    def err(c):
        return ((xe - O.decode(O.encode(xe, c), c)) ** 2).sum(axis=1).mean()
    assert err(cb) < 1.05 * err(cb_ref)
    assert np.isfinite(cb).all()


def test_host_kmeans_with_as_many_centroids_as_points(psc):
    """256 distinct training rows for 256 centroids: every sub-quantizer's codebook must be exactly
    the set of the rows' sub-vectors (each cell holds one point, whose mean is the point), and
    the training set is then quantized without error."""
    rng = np.random.default_rng(21)
    xt = rng.permutation(256 * 64).astype(np.float32).reshape(256, 64)
    idx = psc.Index(64, 8)
    idx.train_pq(xt, iters=3, seed=9)
    cb = idx.get_codebook()
    for j in range(8):
        sub = xt[:, 8 * j:8 * j + 8]
        assert sorted(map(tuple, cb[j])) == sorted(map(tuple, sub)), j
    assert np.array_equal(O.decode(O.encode(xt, cb), cb), xt.astype(np.float64))


def test_annealing_matches_oracle_trajectory(psc):
    """Same counter-based draws, same double-precision objective: the library's annealing
    must end on the oracle's permutation and renumber the codebook the same way."""
    xt = W.sift_like(3000, seed=12, stream=1)
    cb0 = O.train_pq(xt, 8, iters=3, seed=5).astype(np.float32)
    idx = psc.Index(128, 8)
    idx.set_codebook(cb0)
    pi, loss = idx.optimize_index_assignment(n_iter=30_000, seed=77)
    cb_ref, pis_ref, (li, lf) = O.optimize_index_assignment(cb0.astype(np.float64), n_iter=30_000, seed=77)
    assert np.array_equal(pi, pis_ref)
    assert np.allclose(loss[:, 0], li, rtol=1e-12) and np.allclose(loss[:, 1], lf, rtol=1e-9)
    assert np.array_equal(idx.get_codebook(), cb_ref.astype(np.float32))
    for j in range(8):
        assert sorted(pi[j].tolist()) == list(range(256))
    assert np.all(loss[:, 1] < loss[:, 0])


def test_ranking_annealing_matches_oracle_trajectory(psc):
    """The library anneals the ranking loss with sets of centroids as bit masks, the oracle with
    plain loops; same draws and the same double-precision terms, so both walk the same way."""
    xt = W.sift_like(3000, seed=13, stream=1)
    cb0 = O.train_pq(xt, 8, iters=3, seed=5).astype(np.float32)
    idx = psc.Index(128, 8)
    idx.set_codebook(cb0)
    pi, loss = idx.optimize_index_assignment_ranking(n_iter=120, seed=31)
    for j in (0, 5):
        r = O.anneal_ranking(cb0[j].astype(np.float64), n_iter=120, seed=31 + j)
        assert np.array_equal(pi[j], r["pi"]), j
        assert np.isclose(loss[j, 0], r["loss_init"], rtol=1e-12) and np.isclose(loss[j, 1], r["loss_final"], rtol=1e-12)
    # a longer run, checked through the oracle's full evaluation of the loss
    idx.set_codebook(cb0)
    pi, loss = idx.optimize_index_assignment_ranking(n_iter=8000, seed=32)
    for j in (1, 6):
        dmat = O.centroid_distances(cb0[j].astype(np.float64))
        assert sorted(pi[j].tolist()) == list(range(256))
        assert np.isclose(O.polyr_loss(dmat, O.neighbour_ranks(dmat), pi[j]), loss[j, 1], rtol=1e-12)
    assert np.all(loss[:, 1] < loss[:, 0])   # (8000 iterations end at temperature 0.13: still a warm walk)
    assert np.array_equal(idx.get_codebook()[3][pi[3]], cb0[3])     # new row pi[i] = old row i


def test_shape_of_the_comparison_of_methods(psc):
    """The shape of Table 1 (Section 4.2) on synthetic data without cluster structure (one wide
    Gaussian, 32-D, 8-byte codes), recall@100 of the true nearest neighbour:
    ranking by code distance alone -- PQ/binary < PQ/disidx < PolyR/binary <= PolyD/binary;
    filter set to remove >= 95 % of the training pairs, then ADC -- PQ/dual far below PolyR/dual <=
    PolyD/dual <= PQ/ADC.  The index assignments come from the library's host annealing (distance
    loss: the paper's schedule cut to 100k iterations; ranking loss: a faster cooling, 12k
    iterations), everything else from the oracle."""
    kw = dict(seed=31, n_centres=1, sigma=30.0, dim=32)
    xt = W.sift_like(4000, stream=1, **kw)
    xb = W.sift_like(8000, stream=2, **kw) + np.random.default_rng(1).random((8000, 32)).astype(np.float32) * 0.5
    xq = W.sift_like(200, stream=3, **kw)
    cb_pq = O.train_pq(xt, 8, iters=8, seed=3)
    idx = psc.Index(32, 8)
    idx.set_codebook(cb_pq.astype(np.float32))
    idx.optimize_index_assignment(n_iter=100_000, seed=17)
    cb_d = idx.get_codebook().astype(np.float64)
    idx.set_codebook(cb_pq.astype(np.float32))
    _, loss_r = idx.optimize_index_assignment_ranking(n_iter=12_000, t_decay=0.9 ** (1.0 / 50.0), seed=17)
    cb_r = idx.get_codebook().astype(np.float64)
    assert np.all(loss_r[:, 1] < 0.85 * loss_r[:, 0])
    truth = O.exact_knn(xb, xq, 1)[0][:, 0]
    res = {}
    for name, cbk in (("PQ", cb_pq), ("PolyD", cb_d), ("PolyR", cb_r)):
        codes = O.encode(xb, cbk)
        lut = O.build_lut(xq, cbk)
        qc = O.query_codes(lut)
        res[name + "/binary"] = O.recall_at(O.search_by_code_distance(qc, codes, 100, "hamming")[0], truth, 100)
        tc = O.encode(xt[:1500], cbk)
        ht = O.threshold_for_rate(O.hamming_histogram(tc[:100], tc), 0.05)
        r = O.scan(lut, qc, codes, ht, 100)
        assert r["nsurv"].mean() / len(xb) < 0.08
        res[name + "/dual"] = O.recall_at(r["ids"], truth, 100)
        if name == "PQ":
            res["PQ/disidx"] = O.recall_at(O.search_by_code_distance(qc, codes, 100, "disidx")[0], truth, 100)
            res["PQ/ADC"] = O.recall_at(O.scan(lut, qc, codes, 64, 100)["ids"], truth, 100)
    print("recall@100:", {k: round(v, 3) for k, v in res.items()})
    assert res["PQ/binary"] < res["PQ/disidx"] < res["PolyR/binary"] <= res["PolyD/binary"] + 0.03
    assert res["PolyD/binary"] > 3 * res["PQ/binary"]
    assert res["PolyD/dual"] > 3 * res["PQ/dual"] and res["PolyR/dual"] > 2 * res["PQ/dual"]
    assert res["PolyR/dual"] <= res["PolyD/dual"] + 0.03 and res["PolyD/dual"] <= res["PQ/ADC"]
    assert res["PolyD/dual"] > res["PolyD/binary"]      # the second stage repairs the ranking of the survivors


def test_threshold_for_rate_agrees_with_the_oracle():
    """Host-only entry point: same choice as the oracle's rule on random and hand-built histograms."""
    import paper_1609_01882_amd as psc
    rng = np.random.default_rng(12)
    for nbits in (64, 128):
        for _ in range(20):
            hist = rng.integers(0, 1000, size=nbits + 1).astype(np.int64)
            hist[rng.integers(0, nbits + 1, size=nbits // 2)] = 0
            if hist.sum() == 0:
                hist[3] = 1
            for keep in (0.0, 0.001, 0.05, 0.3, 0.999, 1.0):
                assert psc.threshold_for_rate(hist, keep) == O.threshold_for_rate(hist, keep)
    toy = np.array([1, 2, 3, 4], dtype=np.int64)
    assert [psc.threshold_for_rate(toy, r) for r in (0.05, 0.10, 0.30, 0.60, 1.0)] == [-1, 0, 1, 2, 3]
    with pytest.raises(psc.PscError):
        psc.threshold_for_rate(np.zeros(65, dtype=np.int64), 0.5)


def test_workspace_sizes_over_a_grid(psc):
    """The planner (host logic, no GPU): a workspace size for every valid shape of problem, always
    covering status word + shared thresholds + one partial list per query and never more than 1024
    partial lists per query; search and inverted-file workspaces add their tables on top."""
    for m in (8, 16):
        for k in (1, 10, 100, 121, 157, 400, psc.PSC_MAX_K):
            for nq in (1, 4, 5, 16, 17, 1000, 10_000):
                for n in (0, 1, 10_000, 10_000_000, 400_000_000):
                    b = psc.scan_workspace_bytes(m, nq, n, k)
                    assert 256 + 4 * nq + 12 * nq * k <= b <= 1024 + 4 * nq + 256 + 12 * nq * k * 1024, (m, k, nq, n, b)
    idx = psc.Index(128, 8)
    idx.set_codebook(np.zeros((8, 256, 16), np.float32))
    assert idx.search_workspace_bytes(100, 1_000_000, 10) >= psc.scan_workspace_bytes(8, 100, 1_000_000, 10) + 100 * 8 * 1024
    assert idx.knn_graph_workspace_bytes(100_000, 10) > 0
    idx.ivf_set_coarse(np.zeros((50, 128), np.float32))
    small, big = idx.ivf_search_workspace_bytes(1, 8, 10), idx.ivf_search_workspace_bytes(10_000, 8, 10)
    assert 0 < small < big
    # more probes than lists: clipped to the number of lists
    assert idx.ivf_search_workspace_bytes(10, 2000, 10) == idx.ivf_search_workspace_bytes(10, 50, 10)
