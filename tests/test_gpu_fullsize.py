"""Parity at the full workload sizes, in the launch configuration bench.py times: the HIP path
runs the whole batch, the oracle recomputes a sample of the queries one by one (needs an
MI355X; each case takes a few seconds)."""
import numpy as np
import pytest
import torch

import oracle as O
import workloads as W
from gpu_util import RTOL, assert_ivf_topk_matches, assert_topk_matches

pytestmark = pytest.mark.gpu


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _trained_index(psc, cfg, n_train=20_000, sa_iters=100_000):
    xt = cfg.vectors("train", n=n_train, threads=16)
    idx = psc.Index(cfg.dim, cfg.m)
    idx.train_pq(xt, iters=8, seed=cfg.seed)
    idx.optimize_index_assignment(n_iter=sa_iters, seed=cfg.seed)
    return idx


def _encode_db(idx, cfg, n):
    codes = torch.empty((n, cfg.m), dtype=torch.uint8, device="cuda")
    for s in range(0, n, 2_000_000):
        c = min(2_000_000, n - s)
        idx.encode(_dev(cfg.vectors("db", n=c, start=s, threads=16)), out=codes[s:s + c])
    return codes


@pytest.mark.parametrize("name,hts", [("flat64", (16, 24)), ("flat128", (48,))])
def test_flat_full_size(name, hts):
    import paper_1609_01882_amd as psc
    cfg = W.get_config(name)
    idx = _trained_index(psc, cfg)
    codes = _encode_db(idx, cfg, cfg.n_db)
    q_dev = _dev(cfg.vectors("query", threads=16))
    lut, qc = idx.build_lut(q_dev)
    sample = np.sort(np.random.default_rng(5).choice(cfg.n_query, size=48, replace=False))
    sample[:2] = (0, 1)
    sample[-1] = cfg.n_query - 1
    sample = np.unique(sample)
    lut64 = lut[torch.from_numpy(sample).cuda()].cpu().numpy().astype(np.float64)
    qc_h, codes_h = qc.cpu().numpy()[sample], codes.cpu().numpy()
    ws = torch.empty(psc.scan_workspace_bytes(cfg.m, cfg.n_query, cfg.n_db, cfg.k), dtype=torch.uint8, device="cuda")
    for ht in hts:
        print(f"full-size {name} ht={ht}", flush=True)
        ids, d = psc.scan(lut, qc, codes, ht, cfg.k, workspace=ws)
        psc.workspace_status(ws)
        ref = O.scan(lut64, qc_h, codes_h, ht, cfg.k)
        assert_topk_matches(ids.cpu().numpy()[sample], d.cpu().numpy()[sample], ref, lut64, qc_h, codes_h, ht,
                            what=f"{name} ht={ht}")
        # survivor counts of the same queries, bit-exact
        ns = psc.hamming_filter(qc[torch.from_numpy(sample).cuda()].contiguous(), codes, ht)
        assert np.array_equal(ns.cpu().numpy(), ref["nsurv"])
        # whole-batch properties: sorted by (distance, id), ids unique and in range
        ids_h, d_h = ids.cpu().numpy(), d.cpu().numpy()
        assert np.all(np.diff(d_h, axis=1) >= 0) or np.all(np.diff(np.nan_to_num(d_h, posinf=3e38), axis=1) >= 0)
        assert ids_h.max() < cfg.n_db and ids_h.min() >= -1
        assert all(len(set(r[r >= 0].tolist())) == (r >= 0).sum() for r in ids_h[::97])


def test_few_queries_over_400M_codes():
    """The memory-bound launches bench.py times (`small_batch`): 1 and 16 queries over 400M random
    64-bit codes, ht = 20, k = 100 -- 256 database slices per query, which prune with what they
    tell each other.  The oracle re-does the single query and three of the sixteen."""
    import paper_1609_01882_amd as psc
    n, m, k, ht = 400_000_000, 8, 100, 20
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    codes = torch.randint(0, 2 ** 31, (n * m // 4,), dtype=torch.int32, device="cuda", generator=g).view(torch.uint8).view(n, m)
    codes_h = codes.cpu().numpy()
    for nq, sample in ((1, [0]), (16, [0, 7, 15])):
        # queries near stored codes, so that the threshold lets a few thousand codes through
        rows = torch.randint(0, n, (nq,), device="cuda", generator=g)
        qc = codes[rows].clone()
        qc[:, 0] ^= 0x55
        lut = torch.rand((nq, m, 256), device="cuda", generator=g) * 1000.0
        print(f"few queries: nq={nq} over {n} codes", flush=True)
        ids, d = psc.scan(lut, qc, codes, ht, k)
        torch.cuda.synchronize()
        assert "slices=256" in psc.last_scan_route(), psc.last_scan_route()
        lut64, qc_h = lut.cpu().numpy().astype(np.float64)[sample], qc.cpu().numpy()[sample]
        ref = O.scan(lut64, qc_h, codes_h, ht, k)
        assert (ref["nsurv"] > 1000).all()
        assert_topk_matches(ids.cpu().numpy()[sample], d.cpu().numpy()[sample], ref, lut64, qc_h, codes_h, ht,
                            what=f"{nq} queries over 400M codes")


def test_graph_full_size():
    import paper_1609_01882_amd as psc
    cfg = W.get_config("graph")
    idx = _trained_index(psc, cfg)
    x = cfg.vectors("db", threads=16)
    x_dev = _dev(x)
    codes = idx.encode(x_dev)
    ht, k = cfg.hts[0], cfg.k
    ids, d = idx.knn_graph(x_dev, codes, ht, k)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 1, 32767, 32768, cfg.n_db - 1],
                                     np.random.default_rng(3).integers(0, cfg.n_db, 40)]))
    codes_h = codes.cpu().numpy()
    lut64 = idx.build_lut(x_dev[torch.from_numpy(rows).cuda()])[0].cpu().numpy().astype(np.float64)
    ref = O.scan(lut64, codes_h[rows], codes_h, ht, k, skip_id=rows)
    assert_topk_matches(ids.cpu().numpy()[rows], d.cpu().numpy()[rows], ref, lut64, codes_h[rows], codes_h, ht,
                        what="graph full size")
    ids_h = ids.cpu().numpy()
    assert not np.any(ids_h[::1013] == np.arange(cfg.n_db)[::1013, None])


def test_ivf_full_size():
    """The inverted-file workload as configured: 100M vectors in 4096 lists, 64 probes, the 10k-query
    batch, ht = 24, k = 100 -- the launch the benchmark times.  The oracle re-does 24 sampled queries
    over their probed lists on the same decisions (lists, per-list bit strings); every id that
    differs from the oracle's is re-derived from the index."""
    import paper_1609_01882_amd as psc
    from paper_1609_01882_amd.benchmarks._common import build_ivf_workload
    cfg = W.get_config("ivf")
    print("full-size ivf: building 100M lists", flush=True)
    idx, offsets, lcodes, lids, counts = build_ivf_workload(
        psc, cfg, cfg.n_db, torch.device("cuda:0"), coarse_train=200_000, coarse_iters=5, pq_train=20_000,
        pq_iters=8, sa_iters=100_000)
    coarse, cb = idx.ivf_get_coarse(), idx.get_codebook()
    xq = cfg.vectors("query", threads=16)
    ht, k = cfg.hts[0], cfg.k
    print("full-size ivf: search", flush=True)
    ws = torch.empty(idx.ivf_search_workspace_bytes(cfg.n_query, cfg.nprobe, k), dtype=torch.uint8, device="cuda")
    ids, d, probed, qcodes = idx.ivf_search(_dev(xq), cfg.nprobe, ht, k, workspace=ws, want_debug=True)
    psc.workspace_status(ws)
    sample = np.unique(np.concatenate([[0, cfg.n_query - 1], np.random.default_rng(9).integers(0, cfg.n_query, 22)]))
    st = torch.from_numpy(sample).cuda()
    probed_s, qcodes_s = probed[st].cpu().numpy(), qcodes[st].cpu().numpy()
    off_h, lcodes_h, lids_h = offsets.cpu().numpy(), lcodes.cpu().numpy(), lids.cpu().numpy()
    print("full-size ivf: oracle on the sample", flush=True)
    ref = O.ivf_search(xq[sample], cb, coarse, off_h, lcodes_h, lids_h, cfg.nprobe, ht, k,
                       probed_in=probed_s, qcodes_in=qcodes_s)
    # the probed lists are the nearest ones in the oracle's eyes, up to near-ties
    own = O.ivf_search(xq[sample][:4], cb, coarse, off_h, lcodes_h, lids_h, cfg.nprobe, ht, 1, want_coarse=True)
    for q, p in np.argwhere(own["probed"] != probed_s[:4]):
        a, b = own["coarse_d"][q, own["probed"][q, p]], own["coarse_d"][q, probed_s[q, p]]
        assert abs(a - b) <= RTOL * a
    assert_ivf_topk_matches(ids[st].cpu().numpy(), d[st].cpu().numpy(), ref, xq[sample], cb, coarse, off_h, lcodes_h,
                            lids_h, probed_s, qcodes_s, ht, O.build_lut, what="ivf full size")
    # whole-batch properties: sorted, ids in range and unique per row
    ids_h, d_h = ids.cpu().numpy(), d.cpu().numpy()
    assert np.all(np.diff(np.nan_to_num(d_h, posinf=3e38), axis=1) >= 0)
    assert ids_h.max() < cfg.n_db and ids_h.min() >= -1
    assert all(len(set(r[r >= 0].tolist())) == (r >= 0).sum() for r in ids_h[::97])


def test_imi_at_a_million_cells():
    """The inverted multi-index at 1024 x 1024 cells over 10M vectors, 10k-query batch, in the two cap
    settings of Table 2 that the benchmark times (16 cells / 10k codes; 1024 cells / 30k codes): 24
    sampled queries re-done by the oracle on the GPU's decisions, 6 of them also with the oracle's own
    ordering of all 1M cells."""
    import paper_1609_01882_amd as psc
    from paper_1609_01882_amd.benchmarks._common import build_imi_workload
    cfg = W.get_config("ivf")
    kh = 1024
    print("full-size imi: building", flush=True)
    idx, offsets, lcodes, lids, tcodes = build_imi_workload(psc, cfg, 10_000_000, kh, torch.device("cuda:0"),
                                                            coarse_train=200_000, coarse_iters=5, pq_train=20_000,
                                                            pq_iters=8, sa_iters=100_000)
    c1, c2, cb = idx._imi_c1, idx._imi_c2, idx.get_codebook()
    xq = cfg.vectors("query", threads=16)
    off_h, lcodes_h, lids_h = offsets.cpu().numpy(), lcodes.cpu().numpy(), lids.cpu().numpy()
    sample = np.unique(np.concatenate([[0, cfg.n_query - 1], np.random.default_rng(4).integers(0, cfg.n_query, 22)]))
    st = torch.from_numpy(sample).cuda()
    ht, k = 26, cfg.k

    class Centroids:   # cell centroid on demand (1M x 128 floats would do as well; this keeps it small)
        def __getitem__(self, cell):
            return np.concatenate([c1[cell // kh], c2[cell % kh]])

    for max_lists, max_codes in ((16, 10_000), (1024, 30_000)):
        print(f"full-size imi: search {max_lists}/{max_codes}", flush=True)
        ids, d, cells, qcodes = idx.imi_search(_dev(xq), max_lists, max_codes, ht, k, want_debug=True)
        torch.cuda.synchronize()
        cells_s, qcodes_s = cells[st].cpu().numpy(), qcodes[st].cpu().numpy()
        ref = O.imi_search(xq[sample], cb, c1, c2, off_h, lcodes_h, lids_h, max_lists, max_codes, ht, k,
                           cells_in=cells_s, qcodes_in=qcodes_s)
        assert_ivf_topk_matches(ids[st].cpu().numpy(), d[st].cpu().numpy(), ref, xq[sample], cb, Centroids(), off_h,
                                lcodes_h, lids_h, cells_s, qcodes_s, ht, O.build_lut, what=f"imi {max_lists}/{max_codes}")
        own = O.imi_search(xq[sample[:6]], cb, c1, c2, off_h, lcodes_h, lids_h, max_lists, max_codes, ht, k)
        for q, p in np.argwhere(own["cells"] != cells_s[:6]):
            a, b = own["cells"][q, p], cells_s[q, p]
            assert a >= 0 and b >= 0
            da = ((xq[sample[q]].astype(np.float64) - Centroids()[a]) ** 2).sum()
            db = ((xq[sample[q]].astype(np.float64) - Centroids()[b]) ** 2).sum()
            assert abs(da - db) <= RTOL * da
        ids_h = ids.cpu().numpy()
        assert ids_h.max() < 10_000_000 and ids_h.min() >= -1
        assert all(len(set(r[r >= 0].tolist())) == (r >= 0).sum() for r in ids_h[::97])
