"""Parity of the inverted multi-index search (Section 4.3; caption of Table 2) with the oracle
(needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle as O
import workloads as W
from gpu_util import RTOL, assert_ivf_topk_matches

pytestmark = pytest.mark.gpu


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def build_imi(psc, n, k1, k2, seed, m=8, dim=128, noise=0.0):
    """Halves of the coarse quantizer trained by the oracle's k-means (inputs to both sides), residual
    PQ trained by the library, cells assigned and encoded by the library, grouped by a stable sort."""
    rng = np.random.default_rng(seed)
    xt = W.sift_like(5000, seed=seed, stream=1, dim=dim)
    xb = W.sift_like(n, seed=seed, stream=2, dim=dim)
    if noise:
        xb = (xb + rng.random(xb.shape) * noise).astype(np.float32)
    half = dim // 2
    c1, c2 = O.imi_train_coarse(xt, k1, k2, iters=4, seed=1)
    c1, c2 = c1.astype(np.float32), c2.astype(np.float32)
    idx = psc.Index(dim, m)
    idx.imi_set_coarse(c1, c2)
    cell_t, _ = idx.imi_assign_encode(_dev(xt), want_codes=False)
    ct = cell_t.cpu().numpy()
    idx.train_pq(xt - np.concatenate([c1[ct // k2], c2[ct % k2]], axis=1), iters=5, seed=4)
    idx.optimize_index_assignment(n_iter=30_000, seed=5)
    cell, codes = idx.imi_assign_encode(_dev(xb))
    torch.cuda.synchronize()
    order = torch.sort(cell.to(torch.int64), stable=True).indices
    offsets = torch.zeros(k1 * k2 + 1, dtype=torch.int64, device="cuda")
    offsets[1:] = torch.cumsum(torch.bincount(cell.to(torch.int64), minlength=k1 * k2), 0)
    lcodes, lids = codes[order].contiguous(), order.to(torch.int32).contiguous()
    idx.imi_set_lists(offsets, lcodes, lids)
    cc = np.concatenate([np.repeat(c1, k2, axis=0), np.tile(c2, (k1, 1))], axis=1)   # cell centroids, row a*k2+b
    return dict(idx=idx, xb=xb, c1=c1, c2=c2, k2=k2, cc=cc, cb=idx.get_codebook(), cell=cell.cpu().numpy(),
                codes=codes.cpu().numpy(), offsets=offsets.cpu().numpy(), lcodes=lcodes.cpu().numpy(),
                lids=lids.cpu().numpy(), dim=dim, m=m)


@pytest.fixture(scope="module")
def imi():
    import paper_1609_01882_amd as psc
    return psc, build_imi(psc, 60_001, 12, 9, seed=81)


def test_cells_and_residual_codes(imi):
    psc, s = imi
    n = 20_000
    d = ((s["xb"][:n, None, :].astype(np.float64) - s["cc"][None, :, :].astype(np.float64)) ** 2).sum(axis=2)
    ref = d.argmin(axis=1)
    bad = np.flatnonzero(s["cell"][:n] != ref)
    assert len(bad) < 10
    for i in bad:  # only near-ties may fall the other way
        assert abs(d[i, s["cell"][i]] - d[i, ref[i]]) <= RTOL * d[i, ref[i]]
    res = s["xb"][:n].astype(np.float64) - s["cc"][s["cell"][:n]].astype(np.float64)
    assert (O.encode(res, s["cb"]) != s["codes"][:n]).sum() < 20
    assert sorted(s["lids"].tolist()) == list(range(len(s["xb"])))


def _check(fixture, nq, max_lists, max_codes, ht, k, seed=3):
    psc, s = fixture
    idx = s["idx"]
    xq = W.sift_like(nq, seed=81, stream=3, dim=s["dim"])
    ids, d, cells, qcodes = idx.imi_search(_dev(xq), max_lists, max_codes, ht, k, want_debug=True)
    torch.cuda.synchronize()
    ids, d, cells, qcodes = ids.cpu().numpy(), d.cpu().numpy(), cells.cpu().numpy(), qcodes.cpu().numpy()
    # the oracle's own cell order and caps: the same cells in the same order, up to near-ties of the sums
    own = O.imi_search(xq, s["cb"], s["c1"], s["c2"], s["offsets"], s["lcodes"], s["lids"], max_lists, max_codes, ht, k)
    dc = ((xq[:, None, :].astype(np.float64) - s["cc"][None, :, :].astype(np.float64)) ** 2).sum(axis=2)
    diff = np.argwhere(own["cells"] != cells)
    for q, p in diff:
        a, b = own["cells"][q, p], cells[q, p]
        assert a >= 0 and b >= 0, (q, p, a, b)
        assert abs(dc[q, a] - dc[q, b]) <= RTOL * dc[q, a]
    assert len(diff) <= max(2, 0.005 * cells.size)
    # same decisions (cells, bit strings) -> same survivors, ids and distances
    ref = O.imi_search(xq, s["cb"], s["c1"], s["c2"], s["offsets"], s["lcodes"], s["lids"], max_lists, max_codes, ht, k,
                       cells_in=cells, qcodes_in=qcodes)
    assert_ivf_topk_matches(ids, d, ref, xq, s["cb"], s["cc"], s["offsets"], s["lcodes"], s["lids"], cells, qcodes, ht,
                            O.build_lut, what=f"imi nq={nq} lists={max_lists} codes={max_codes} ht={ht} k={k}")
    own_q = O.imi_search(xq, s["cb"], s["c1"], s["c2"], s["offsets"], s["lcodes"], s["lids"], max_lists, max_codes, ht, k,
                         cells_in=cells)
    assert (own_q["nsurv"] != ref["nsurv"]).sum() <= max(1, 0.1 * nq)


@pytest.mark.parametrize("nq,max_lists,max_codes,ht,k", [
    (37, 16, 0, 24, 10), (37, 16, 3000, 64, 100), (1, 4, 0, 20, 10), (300, 108, 0, 28, 100), (5, 200, 0, 30, 300),
    (64, 1, 0, 26, 5), (20, 30, 1, 24, 10), (33, 50, 20_000, 0, 1), (10, 1024, 25_000, 22, 1000)])
def test_imi_search_matches_oracle(imi, nq, max_lists, max_codes, ht, k):
    """Caps on cells and on codes in every combination (none, one binding, both), more cells asked for
    than exist, a single query and a batch, k beyond the survivors."""
    _check(imi, nq, max_lists, max_codes, ht, k)


@pytest.fixture(scope="module")
def imi_many_cells():
    import paper_1609_01882_amd as psc
    return psc, build_imi(psc, 50_000, 200, 180, seed=82)


@pytest.mark.parametrize("nq,max_lists,max_codes,ht,k", [(25, 16, 0, 24, 10), (40, 1024, 10_000, 26, 100), (7, 300, 500, 64, 50),
                                                         (1, 1024, 0, 24, 100), (60, 200, 60, 26, 10), (60, 1024, 90, 64, 20),
                                                         (30, 65, 80, 24, 10), (30, 64, 80, 24, 10)])
def test_imi_with_36000_cells(imi_many_cells, nq, max_lists, max_codes, ht, k):
    """Cells of one or two codes, most of them empty: the regime of a real multi-index (here 36000
    cells for 50000 vectors), with up to 1024 cells per query and the cap on codes binding.  Caps of
    60 to 90 codes are reached after about 64 cells: by some queries within the first pass over the
    cell order, by others only in the full one."""
    _check(imi_many_cells, nq, max_lists, max_codes, ht, k)


def test_imi_settings_drawn_at_random(imi_many_cells):
    """Caps, threshold, k and batch size drawn (seeded) from the values around which the library
    changes what it does: 64 and 256 cells (the passes over the cell order), 256 queries (several
    workgroups per query up to there), k beyond one pool."""
    rng = np.random.default_rng(4242)
    for _ in range(14):
        max_lists = int(rng.choice([1, 3, 16, 63, 64, 65, 255, 256, 257, 600, 1024]))
        max_codes = int(rng.choice([0, 1, 30, 80, 200, 1000, 5000, 40_000]))
        ht = int(rng.choice([0, 16, 24, 28, 40, 64]))
        k = int(rng.choice([1, 10, 100, 300, 1000]))
        nq = int(rng.choice([1, 3, 20, 64, 256, 257]))
        print(f"imi drawn: lists={max_lists} codes={max_codes} ht={ht} k={k} nq={nq}", flush=True)
        _check(imi_many_cells, nq, max_lists, max_codes, ht, k)


def test_imi_with_128_bit_codes():
    import paper_1609_01882_amd as psc
    s = build_imi(psc, 30_000, 10, 11, seed=83, m=16)
    _check((psc, s), 21, 20, 0, 50, 20)
    _check((psc, s), 3, 110, 4000, 128, 10)


def test_imi_in_another_dimension_without_exact_ties():
    """64-D vectors with a little noise (no exactly tied cell distances), 4 sub-quantizers per half."""
    import paper_1609_01882_amd as psc
    s = build_imi(psc, 30_000, 17, 13, seed=84, dim=64, noise=0.7)
    _check((psc, s), 50, 25, 2500, 26, 30)


def test_imi_with_more_dimensions_than_threads():
    """384-D vectors (48 dimensions per sub-quantizer, more dimensions than a workgroup has threads):
    the residual is then put together in several turns per thread."""
    import paper_1609_01882_amd as psc
    s = build_imi(psc, 20_000, 11, 9, seed=85, dim=384, noise=0.7)
    _check((psc, s), 30, 20, 3000, 28, 20)
    _check((psc, s), 300, 8, 0, 64, 10)


def test_one_centroid_in_the_second_half_is_the_inverted_file():
    """K2 = 1: the multi-index is an inverted file over the first-half centroids; the library's two
    searches agree on lists and results (distances to float32 rounding: different table kernels)."""
    import paper_1609_01882_amd as psc
    xt = W.sift_like(4000, seed=85, stream=1)
    xb = W.sift_like(30_000, seed=85, stream=2)
    xq = W.sift_like(30, seed=85, stream=3)
    c1, c2 = O.imi_train_coarse(xt, 20, 1, iters=4, seed=2)
    c1, c2 = c1.astype(np.float32), c2.astype(np.float32)
    coarse = np.concatenate([c1, np.repeat(c2, 20, axis=0)], axis=1)
    idx = psc.Index(128, 8)
    idx.imi_set_coarse(c1, c2)
    idx.ivf_set_coarse(coarse)
    lt, _ = idx.ivf_assign_encode(_dev(xt), want_codes=False)
    idx.train_pq(xt - coarse[lt.cpu().numpy()], iters=4, seed=1)
    cell, codes = idx.imi_assign_encode(_dev(xb))
    list_no, codes2 = idx.ivf_assign_encode(_dev(xb))
    assert (cell != list_no).float().mean() < 1e-3 and (codes != codes2).float().mean() < 1e-3
    order = torch.sort(cell.to(torch.int64), stable=True).indices
    offsets = torch.zeros(21, dtype=torch.int64, device="cuda")
    offsets[1:] = torch.cumsum(torch.bincount(cell.to(torch.int64), minlength=20), 0)
    lcodes, lids = codes[order].contiguous(), order.to(torch.int32).contiguous()
    idx.imi_set_lists(offsets, lcodes, lids)
    idx.ivf_set_lists(offsets, lcodes, lids)
    a_ids, a_d, cells, _ = idx.imi_search(_dev(xq), 5, 0, 26, 20, want_debug=True)
    b_ids, b_d, probed, _ = idx.ivf_search(_dev(xq), 5, 26, 20, want_debug=True)
    torch.cuda.synchronize()
    assert (cells != probed).float().mean() < 0.02
    same = (cells == probed).all(dim=1)
    assert torch.allclose(a_d[same], b_d[same], rtol=1e-5, atol=0.0)
    assert (a_ids[same] == b_ids[same]).float().mean() > 0.97


def test_imi_argument_errors():
    import paper_1609_01882_amd as psc
    idx = psc.Index(128, 8)
    q = torch.zeros((2, 128), device="cuda")
    with pytest.raises(psc.PscError):
        idx.imi_search(q, 16, 0, 24, 10)                      # no coarse quantizer
    idx.imi_set_coarse(np.zeros((3, 64), np.float32), np.zeros((2, 64), np.float32))
    idx.set_codebook(np.zeros((8, 256, 16), np.float32))
    with pytest.raises(psc.PscError):
        idx.imi_search(q, 16, 0, 24, 10)                      # no lists
    codes = torch.zeros((10, 8), dtype=torch.uint8, device="cuda")
    ids = torch.arange(10, dtype=torch.int32, device="cuda")
    with pytest.raises(psc.PscError):
        idx.imi_set_lists(torch.tensor([0, 4, 8, 9, 9, 9, 9], dtype=torch.int64, device="cuda"), codes, ids)
    idx.imi_set_lists(torch.tensor([0, 4, 4, 4, 10, 10, 10], dtype=torch.int64, device="cuda"), codes, ids)
    with pytest.raises(psc.PscError):
        idx.imi_search(q, 2000, 0, 24, 10)                    # more than 1024 cells per query
    out = idx.imi_search(q, 6, 0, 64, 12)
    torch.cuda.synchronize()
    assert sorted(out[0][0][:10].tolist()) == list(range(10)) and out[0][0][10:].tolist() == [-1, -1]


@pytest.mark.parametrize("spread,sigma,direct", [(300.0, 10.0, False), (4000.0, 10.0, True)])
def test_imi_distances_when_the_half_centroids_lie_far_apart(spread, sigma, direct):
    """The 1e-5 bound away from the comfortable data scale, as for the inverted file: half-centroids
    uniform in [0, spread]^64 with the vectors within sigma of a cell centroid.  Below the rule's
    limit the cell tables are added up from the query's and the half-centroids' shares, above it they
    are built by direct differences; both agree with the float64 oracle."""
    import paper_1609_01882_amd as psc
    rng = np.random.default_rng(int(spread))
    k1, k2, n, nq = 9, 7, 20_000, 40
    c1 = (rng.random((k1, 64)) * spread).astype(np.float32)
    c2 = (rng.random((k2, 64)) * spread).astype(np.float32)

    def draw(count):
        a, b = rng.integers(0, k1, size=count), rng.integers(0, k2, size=count)
        return (np.concatenate([c1[a], c2[b]], axis=1) + rng.normal(0, sigma, size=(count, 128))).astype(np.float32)
    xt, xb, xq = draw(4000), draw(n), draw(nq)
    idx = psc.Index(128, 8)
    idx.imi_set_coarse(c1, c2)
    ct = idx.imi_assign_encode(_dev(xt), want_codes=False)[0].cpu().numpy()
    idx.train_pq(xt - np.concatenate([c1[ct // k2], c2[ct % k2]], axis=1), iters=5, seed=4)
    cell, codes = idx.imi_assign_encode(_dev(xb))
    order = torch.sort(cell.to(torch.int64), stable=True).indices
    offsets = torch.zeros(k1 * k2 + 1, dtype=torch.int64, device="cuda")
    offsets[1:] = torch.cumsum(torch.bincount(cell.to(torch.int64), minlength=k1 * k2), 0)
    lcodes, lids = codes[order].contiguous(), order.to(torch.int32).contiguous()
    idx.imi_set_lists(offsets, lcodes, lids)
    cc = np.concatenate([np.repeat(c1, k2, axis=0), np.tile(c2, (k1, 1))], axis=1)
    cb, off_h, lc_h, li_h = idx.get_codebook(), offsets.cpu().numpy(), lcodes.cpu().numpy(), lids.cpu().numpy()
    for max_lists, ht, k in ((6, 26, 20), (3, 64, 50)):
        ids, d, cells, qcodes = idx.imi_search(_dev(xq), max_lists, 0, ht, k, want_debug=True)
        torch.cuda.synchronize()
        cells, qcodes = cells.cpu().numpy(), qcodes.cpu().numpy()
        ref = O.imi_search(xq, cb, c1, c2, off_h, lc_h, li_h, max_lists, 0, ht, k, cells_in=cells, qcodes_in=qcodes)
        assert_ivf_topk_matches(ids.cpu().numpy(), d.cpu().numpy(), ref, xq, cb, cc, off_h, lc_h, li_h, cells, qcodes, ht,
                                O.build_lut, what=f"imi spread {spread}")
        own = O.imi_search(xq, cb, c1, c2, off_h, lc_h, li_h, max_lists, 0, ht, k)
        assert (own["cells"] != cells).mean() < 0.02
    # which path ran (the rule's ratio is about 0.03 x spread for sigma = 10, its limit 16)
    assert psc.last_scan_route().split()[0] == ("imi_scan_kernel+direct-tables" if direct else "imi_scan_kernel")
