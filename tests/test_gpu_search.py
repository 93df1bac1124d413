"""Parity of tables, encoding and the whole flat search with the oracle on the trained,
SIFT-like workload (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle as O
import workloads as W
from gpu_util import RTOL, assert_topk_matches

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def setup():
    import paper_1609_01882_amd as psc
    out = {}
    for m in (8, 16):
        xt = W.sift_like(4000, seed=60 + m, stream=1)
        xb = W.sift_like(60_001, seed=60 + m, stream=2)
        xq = W.sift_like(50, seed=60 + m, stream=3)
        idx = psc.Index(128, m)
        idx.train_pq(xt, iters=5, seed=1)
        idx.optimize_index_assignment(n_iter=30_000, seed=2)
        out[m] = dict(idx=idx, cb=idx.get_codebook(), xb=xb, xq=xq)
    out["psc"] = psc
    return out


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("m", [8, 16])
def test_tables_and_query_codes(setup, m):
    s = setup[m]
    lut, qc = s["idx"].build_lut(_dev(s["xq"]))
    torch.cuda.synchronize()
    lut, qc = lut.cpu().numpy(), qc.cpu().numpy()
    ref = O.build_lut(s["xq"], s["cb"])
    # The tables come from the expansion |q'|^2 - 2 q'.c' + |c'|^2 in float32 on the matrix
    # cores, entries that cancel to less than 1/16 of those terms being redone by direct
    # differences: every entry is within the path's 1e-5 of its own value.
    allow = RTOL * ref
    assert np.all(np.abs(lut - ref) <= allow), np.max(np.abs(lut - ref) / allow)
    # ADC sums built from these tables stay within the 1e-5 relative bound of the path
    codes = W.random_codes(4000, m, seed=3)
    got = sum(lut[:, j, codes[:, j]].astype(np.float64) for j in range(m))
    want = sum(ref[:, j, codes[:, j]] for j in range(m))
    assert np.max(np.abs(got - want) / want) < RTOL / 10
    # the query code is the arg-min of the float32 table row (lowest index on ties) ...
    assert np.array_equal(qc, lut.argmin(axis=2).astype(np.uint8))
    # ... and a valid code in the oracle's eyes: its entry is within tolerance of the row minimum
    pick = np.take_along_axis(ref, qc[:, :, None].astype(np.int64), axis=2)[:, :, 0]
    assert np.all(pick <= ref.min(axis=2) * (1 + 2 * RTOL))
    assert (qc == O.query_codes(ref)).mean() > 0.999


@pytest.mark.parametrize("m", [8, 16])
def test_encode(setup, m):
    s = setup[m]
    codes = s["idx"].encode(_dev(s["xb"])).cpu().numpy()
    ref = O.encode(s["xb"][:20_000], s["cb"])
    got = codes[:20_000]
    bad = np.argwhere(got != ref)
    assert len(bad) < 20  # only near-ties may differ
    dsub = 128 // m
    for i, j in bad:
        v = s["xb"][i, j * dsub:(j + 1) * dsub].astype(np.float64)
        da = ((v - s["cb"][j, got[i, j]]) ** 2).sum()
        db = ((v - s["cb"][j, ref[i, j]]) ** 2).sum()
        assert abs(da - db) <= RTOL * db
    s["codes"] = codes


@pytest.mark.parametrize("m", [8, 16])
def test_whole_search_matches_oracle(setup, m):
    s = setup[m]
    idx = s["idx"]
    if "codes" not in s:
        s["codes"] = idx.encode(_dev(s["xb"])).cpu().numpy()
    codes = s["codes"]
    q_dev, c_dev = _dev(s["xq"]), _dev(codes)
    lut, qc = idx.build_lut(q_dev)
    lut64, qc = lut.cpu().numpy().astype(np.float64), qc.cpu().numpy()
    nb = 8 * m
    for ht, k in ((nb // 4, 10), (nb * 3 // 8, 10), (nb * 3 // 8, 100), (nb // 2, 100), (nb, 100)):
        print(f"search m={m} ht={ht} k={k}", flush=True)
        ids, d = idx.search(q_dev, c_dev, ht, k)
        torch.cuda.synchronize()
        ref = O.scan(lut64, qc, codes, ht, k)
        assert_topk_matches(ids.cpu().numpy(), d.cpu().numpy(), ref, lut64, qc, codes, ht, what=f"m={m} ht={ht}")
        # and against the oracle's own double-precision tables: same ranking up to tolerance ties
        ref2 = O.search_flat(s["xq"], s["cb"], codes, ht, k)
        same_codes = np.all(O.query_codes(O.build_lut(s["xq"], s["cb"])) == qc, axis=1)
        assert same_codes.mean() > 0.9
        gd = d.cpu().numpy()[same_codes]
        fin = np.isfinite(ref2["dists"][same_codes])
        assert np.allclose(gd[fin], ref2["dists"][same_codes][fin], rtol=RTOL)


def test_tiny_workload_as_configured():
    """The smallest named workload, whole: 10k training vectors, product quantizer with optimised
    index assignment (the paper's annealing constants), 100 000 database vectors, 100 queries,
    ht = 24, k = 10 -- every query checked against the oracle, on the library's tables and on the
    oracle's own double-precision path from the raw vectors; recall@10 of both sides coincides."""
    import paper_1609_01882_amd as psc
    cfg = W.get_config("tiny")
    assert (cfg.n_train, cfg.n_db, cfg.n_query, cfg.hts, cfg.k) == (10_000, 100_000, 100, (24,), 10)
    xt, xb, xq = cfg.vectors("train"), cfg.vectors("db"), cfg.vectors("query")
    idx = psc.Index(cfg.dim, cfg.m)
    idx.train_pq(xt, iters=20, seed=cfg.seed)
    idx.optimize_index_assignment(seed=cfg.seed)
    cb = idx.get_codebook()
    ht, k = cfg.hts[0], cfg.k
    codes = idx.encode(_dev(xb))
    ids, d = idx.search(_dev(xq), codes, ht, k)
    lut, qc = idx.build_lut(_dev(xq))
    torch.cuda.synchronize()
    ids, d, codes_h = ids.cpu().numpy(), d.cpu().numpy(), codes.cpu().numpy()
    lut64, qc = lut.cpu().numpy().astype(np.float64), qc.cpu().numpy()
    # same tables and bit strings on both sides: survivor counts exact, ids and distances to the bar
    ref = O.scan(lut64, qc, codes_h, ht, k)
    assert_topk_matches(ids, d, ref, lut64, qc, codes_h, ht, what="tiny")
    ns = psc.hamming_filter(_dev(qc), codes, ht)
    assert np.array_equal(ns.cpu().numpy(), ref["nsurv"])
    # the oracle's own path from the raw vectors (its encoding, its tables, its query codes)
    ref_codes = O.encode(xb, cb)
    bad = np.argwhere(ref_codes != codes_h)
    assert len(bad) < 50
    dsub = cfg.dim // cfg.m
    for i, j in bad:  # only near-ties may be encoded differently
        v = xb[i, j * dsub:(j + 1) * dsub].astype(np.float64)
        da, db = ((v - cb[j, codes_h[i, j]]) ** 2).sum(), ((v - cb[j, ref_codes[i, j]]) ** 2).sum()
        assert abs(da - db) <= RTOL * db
    own = O.search_flat(xq, cb, codes_h, ht, k)
    same = np.all(O.query_codes(O.build_lut(xq, cb)) == qc, axis=1)
    assert same.mean() >= 0.95
    fin = np.isfinite(own["dists"][same])
    assert np.allclose(d[same][fin], own["dists"][same][fin], rtol=RTOL)
    assert np.array_equal(np.isfinite(d[same]), fin)
    truth = O.exact_knn(xb, xq, 1)[0][:, 0]
    r_gpu, r_orc = O.recall_at(ids, truth, 10), O.recall_at(ref["ids"], truth, 10)
    print(f"tiny: recall@10 gpu {r_gpu:.3f} oracle {r_orc:.3f}, survivors/query {ref['nsurv'].mean():.0f}", flush=True)
    assert r_gpu == r_orc


@pytest.mark.parametrize("m,spread,sigma", [(8, 3000.0, 10.0), (16, 30000.0, 2.0), (8, 100.0, 15.0)])
def test_tables_when_centroids_lie_far_apart(m, spread, sigma):
    """The table kernel's expansion |q'|^2 - 2 q'.c' + |c'|^2 cancels badly for a centroid close to
    the query when the centroids are spread far wider than that distance; such entries are redone
    by direct differences, so every entry -- small ones included -- is within 1e-5 of its own
    value, on clustered centroids 30 to 10000 times farther apart than the query is from the
    nearest one, and the query code is the oracle's except on near-ties."""
    import paper_1609_01882_amd as psc
    rng = np.random.default_rng(int(spread) + m)
    dsub = 128 // m
    centres = rng.random((40, 128)) * spread
    cb = np.empty((m, 256, dsub), np.float32)
    for j in range(m):   # centroids scattered around the 40 cluster centres of each sub-space
        cb[j] = centres[rng.integers(0, 40, size=256), j * dsub:(j + 1) * dsub] + rng.normal(0, sigma, size=(256, dsub))
    xq = (centres[rng.integers(0, 40, size=300)] + rng.normal(0, sigma, size=(300, 128))).astype(np.float32)
    idx = psc.Index(128, m)
    idx.set_codebook(cb)
    lut, qc = idx.build_lut(_dev(xq))
    torch.cuda.synchronize()
    lut, qc = lut.cpu().numpy(), qc.cpu().numpy()
    ref = O.build_lut(xq, cb)
    err = np.abs(lut - ref) / np.maximum(ref, 1e-30)
    print(f"tables m={m} spread={spread}: max rel err {err.max():.2e}, row max/min up to "
          f"{(ref.max(axis=2) / ref.min(axis=2)).max():.1e}", flush=True)
    assert err.max() <= RTOL
    assert np.array_equal(qc, lut.argmin(axis=2).astype(np.uint8))
    pick = np.take_along_axis(ref, qc[:, :, None].astype(np.int64), axis=2)[:, :, 0]
    assert np.all(pick <= ref.min(axis=2) * (1 + 2 * RTOL))
