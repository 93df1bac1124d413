"""Parity of the fused HIP scan with the CPU oracle, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle as O
import workloads as W
from gpu_util import RTOL, assert_topk_matches

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def psc():
    import paper_1609_01882_amd as p
    assert torch.cuda.is_available()
    return p


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _rand_problem(m, n, nq, seed, lut_kind):
    rng = np.random.default_rng(seed)
    codes = W.random_codes(n, m, seed=seed)
    # query codes near some database codes so that low thresholds still see survivors
    qcodes = codes[rng.integers(0, max(n, 1), size=nq)].copy() if n > 0 else W.random_codes(nq, m, seed + 1)
    flip = rng.integers(0, 256, size=qcodes.shape).astype(np.uint8) & rng.integers(0, 256, size=qcodes.shape).astype(np.uint8)
    qcodes ^= flip
    if lut_kind == "int":      # few small integers: sums exact in float32, many exact ties
        lut = rng.integers(0, 4, size=(nq, m, 256)).astype(np.float32)
    else:
        lut = (rng.random(size=(nq, m, 256)) * 1000.0).astype(np.float32)
    return codes, qcodes, lut


def _run(psc, lut, qcodes, codes, ht, k):
    ids, d = psc.scan(_dev(lut), _dev(qcodes), _dev(codes), ht, k)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), d.cpu().numpy()


@pytest.mark.parametrize("m,n,nq,k,lut_kind", [
    (8, 100_003, 37, 10, "float"),      # ragged tail (odd n), ragged query tile
    (8, 100_003, 37, 100, "int"),       # exact ties: ids must match exactly
    (8, 4096, 16, 100, "float"),
    (8, 70_001, 5, 1, "float"),
    (16, 50_001, 19, 10, "float"),
    (16, 50_001, 19, 100, "int"),
    (8, 30_000, 3, 300, "int"),         # k > 128: smaller query tile
    (16, 20_000, 9, 1024, "float"),     # maximum k
    (8, 60_001, 1, 100, "float"),       # small batches take narrower query tiles
    (8, 45_003, 8, 10, "int"),
    (16, 33_001, 2, 100, "int"),
    (16, 40_001, 7, 10, "float"),
])
def test_scan_random_codes(psc, m, n, nq, k, lut_kind):
    codes, qcodes, lut = _rand_problem(m, n, nq, seed=100 + m + k, lut_kind=lut_kind)
    nb = 8 * m
    for ht in sorted({0, nb // 4, nb * 3 // 8, nb // 2 - 4, nb // 2, nb, nb + 50}):
        print(f"case m={m} n={n} nq={nq} k={k} lut={lut_kind} ht={ht}", flush=True)
        got_ids, got_d = _run(psc, lut, qcodes, codes, ht, k)
        ref = O.scan(lut.astype(np.float64), qcodes, codes, ht, k)
        nd = assert_topk_matches(got_ids, got_d, ref, lut.astype(np.float64), qcodes, codes, min(ht, nb),
                                 what=f"m={m} ht={ht} k={k}")
        if lut_kind == "int":
            assert nd == 0 and np.array_equal(got_d[ref["ids"] >= 0], ref["dists"][ref["ids"] >= 0])


@pytest.mark.parametrize("route", ["mfma", "popcount"])
@pytest.mark.parametrize("n,nq,k,lut_kind", [
    (100_003, 37, 10, "float"),     # ragged last block (n % 128 = 35), ragged query tile (37 = 2 * 16 + 5)
    (100_003, 37, 100, "int"),      # exact ties: ids must match exactly
    (65_536 + 127, 160, 136, "int"),  # the largest k of the 16-query tile
    (9_000, 17, 5, "float"),        # barely more than one tile of queries, one slice
    (300_001, 9, 10, "int"),        # the fewest queries the matrix-core route takes: many slices
    (50_000, 16, 100, "float"),     # exactly one full tile
    (1_000_001, 48, 20, "float"),   # several slices per query tile
])
def test_both_filter_routes(psc, force_route, route, n, nq, k, lut_kind):
    """The Hamming test runs either as xor/popcount or on the matrix cores; the library picks by
    shape and threshold.  Here each route is forced in turn (psc_set_filter_route) on 64-bit codes
    with 9 queries or more and must give the oracle's result at every threshold, including
    those the rule would hand to the other route."""
    force_route(route)
    codes, qcodes, lut = _rand_problem(8, n, nq, seed=900 + k, lut_kind=lut_kind)
    for ht in (0, 9, 16, 22, 24, 27, 29, 30, 33):
        print(f"case route={route} n={n} nq={nq} k={k} ht={ht}", flush=True)
        got_ids, got_d = _run(psc, lut, qcodes, codes, ht, k)
        # the library says which kernel it launched: the forced filter below the dense route's thresholds
        took = psc.last_scan_route().split()[0]
        assert took == ("adc_kernel+filter" if ht >= 30 else "scan_mfma_kernel" if route == "mfma" else "scan_kernel"), took
        ref = O.scan(lut.astype(np.float64), qcodes, codes, ht, k)
        nd = assert_topk_matches(got_ids, got_d, ref, lut.astype(np.float64), qcodes, codes, ht,
                                 what=f"route={route} ht={ht} k={k}")
        if lut_kind == "int":
            assert nd == 0 and np.array_equal(got_d[ref["ids"] >= 0], ref["dists"][ref["ids"] >= 0])


def test_survivor_set_on_the_matrix_cores(psc, force_route):
    """k above the number of survivors: the matrix-core route lists exactly the survivor set, for
    thresholds on both sides of every bit count the +-1 dot product can take near them."""
    force_route("mfma")
    codes, qcodes, lut = _rand_problem(8, 40_000, 33, seed=77, lut_kind="float")
    for ht in (17, 18, 19, 20):
        ref = O.scan(lut.astype(np.float64), qcodes, codes, ht, 136, want_bitmap=True)
        got_ids, _ = _run(psc, lut, qcodes, codes, ht, 136)
        for q in range(33):
            if ref["nsurv"][q] <= 136:
                assert sorted(got_ids[q][got_ids[q] >= 0].tolist()) == np.flatnonzero(ref["bitmap"][q]).tolist()


@pytest.mark.parametrize("route", ["mfma", "popcount"])
def test_nested_prefix_patterns_at_every_threshold(psc, force_route, route):
    """Database row r = the first r bits set (r = 0..64, repeated to fill several blocks), query q =
    the first 3q bits set: their Hamming distance is |r - 3q| exactly, so the survivor set at every
    threshold is known in closed form.  Both filters at every threshold they serve, and the dense
    route, which tests only the pairs that beat the k-th best, at the thresholds above (30 and
    more); the table makes the distance itself the score."""
    force_route(route)
    m, reps, nq = 8, 7, 20
    def prefix(r):
        c = np.zeros(m, np.uint8)
        full, rem = divmod(r, 8)
        c[:full] = 0xFF
        if rem:
            c[full] = (1 << rem) - 1
        return c
    rows = np.array([r for _ in range(reps) for r in range(65)])
    codes = np.stack([prefix(r) for r in rows])
    qbits = np.array([3 * q for q in range(nq)])
    qc = np.stack([prefix(b) for b in qbits])
    lut = np.zeros((nq, m, 256), np.float32)
    pc = np.array([bin(v).count("1") for v in range(256)], np.float32)
    for q in range(nq):  # score = Hamming distance to the query code: sum over bytes of popcount(byte xor query byte)
        for j in range(m):
            lut[q, j] = pc[np.arange(256) ^ int(qc[q, j])]
    k = 136
    for ht in range(0, 36):
        ids, d = _run(psc, lut, qc, codes, ht, k)
        for q in range(nq):
            want = np.flatnonzero(np.abs(rows - qbits[q]) <= ht)
            got = ids[q][ids[q] >= 0]
            if len(want) <= k:
                assert sorted(got.tolist()) == want.tolist(), (route, ht, q)
            else:
                assert len(got) == k
            assert np.array_equal(d[q][: len(got)], np.abs(rows[got] - qbits[q]).astype(np.float32)), (route, ht, q)


@pytest.mark.parametrize("route", ["mfma", "popcount"])
def test_whole_and_sliced_query_tiles_in_one_launch(psc, force_route, route):
    """More query tiles than workgroups run at a time: the tiles of the whole rounds scan the
    database in one piece, those of the last partial round in slices.  Queries from both regions
    (and the last, ragged tile) against the oracle."""
    force_route(route)
    n, nq, k = 150_011, 4100 + 13, 20
    codes, qcodes, lut = _rand_problem(8, n, nq, seed=4242, lut_kind="float")
    sel = np.array([0, 1, 15, 16, 2047, 4079, 4080, 4095, 4096, 4097, 4111, 4112])
    for ht in (14, 22):
        got_ids, got_d = _run(psc, lut, qcodes, codes, ht, k)
        ref = O.scan(lut[sel].astype(np.float64), qcodes[sel], codes, ht, k)
        assert_topk_matches(got_ids[sel], got_d[sel], ref, lut[sel].astype(np.float64), qcodes[sel], codes, ht,
                            what=f"two regions route={route} ht={ht}")
        # all queries: as many results as the (separately tested) filter counts survivors, up to k
        ns = psc.hamming_filter(_dev(qcodes), _dev(codes), ht)
        torch.cuda.synchronize()
        assert got_ids.max() < n
        assert np.array_equal((got_ids >= 0).sum(axis=1), np.minimum(ns.cpu().numpy(), k))


def test_many_slices_for_few_queries(psc):
    """Two queries over 3M codes: 256 database slices, whose partial lists the merge takes four to a lane."""
    codes, qcodes, lut = _rand_problem(8, 3_000_001, 2, seed=321, lut_kind="float")
    for ht, k in ((22, 10), (64, 3)):
        got_ids, got_d = _run(psc, lut, qcodes, codes, ht, k)
        ref = O.scan(lut.astype(np.float64), qcodes, codes, ht, k)
        assert_topk_matches(got_ids, got_d, ref, lut.astype(np.float64), qcodes, codes, ht, what=f"many slices ht={ht}")


@pytest.mark.parametrize("case", ["all tied", "best in one slice", "wide range"])
@pytest.mark.parametrize("nq,k", [(1, 100), (3, 7), (12, 1), (5, 640)])
def test_what_the_slices_tell_each_other_costs_no_result(psc, case, nq, k):
    """Queries cut into many slices prune with a bound taken from the other slices' lists (the
    r-th best of each, and the value enough of them have reached).  Where that bound equals the
    k-th distance (everything tied), where one slice holds the whole answer, and where distances
    span sixty binary orders of magnitude (the bound is rounded up in the float's bits), the result
    is still the oracle's."""
    n, m = 1_200_007, 8
    rng = np.random.default_rng(900 + k)
    codes, qcodes, lut = _rand_problem(m, n, nq, seed=901 + k, lut_kind="int")
    if case == "all tied":
        lut[:] = 2.0
    elif case == "best in one slice":
        # the last 2000 codes are the only ones with small distances: byte 0 below 16 there only
        codes[:, 0] |= 16
        codes[-2000:, 0] &= 15
        lut[:, 0, :16] = 0.0
        lut[:, 0, 16:] = 50.0
    else:
        lut = np.exp2(rng.uniform(-30.0, 30.0, size=(nq, m, 256))).astype(np.float32)
    for ht in (26, 64):
        got_ids, got_d = _run(psc, lut, qcodes, codes, ht, k)
        ref = O.scan(lut.astype(np.float64), qcodes, codes, ht, k)
        nd = assert_topk_matches(got_ids, got_d, ref, lut.astype(np.float64), qcodes, codes, ht,
                                 what=f"{case} nq={nq} k={k} ht={ht}")
        if case != "wide range":
            assert nd == 0


@pytest.mark.parametrize("nq,n,k,lut_kind", [(1, 3_000_001, 100, "int"), (3, 1_000_003, 64, "int"),
                                             (8, 400_009, 128, "float"), (2, 70_001, 1024, "int"),
                                             (1, 300, 500, "int")])
def test_selecting_merge_for_a_handful_of_queries(psc, nq, n, k, lut_kind):
    """A handful of queries (up to 32, or 512 with many lists each) and k >= 64: the partial lists of the slices are merged by a workgroup that
    selects the k smallest (distance, id) pairs.  Integer tables put hundreds of entries at the
    k-th distance, so the last place is decided by the id; short databases leave padding."""
    codes, qcodes, lut = _rand_problem(8, n, nq, seed=77 + k, lut_kind=lut_kind)
    for ht in (24, 64):
        got_ids, got_d = _run(psc, lut, qcodes, codes, ht, k)
        ref = O.scan(lut.astype(np.float64), qcodes, codes, ht, k)
        nd = assert_topk_matches(got_ids, got_d, ref, lut.astype(np.float64), qcodes, codes, ht, what=f"nq={nq} k={k} ht={ht}")
        if lut_kind == "int":
            assert nd == 0  # exact sums: ties must resolve exactly as in the oracle


@pytest.mark.parametrize("m,n,k,lut_kind", [(8, 2_000_003, 100, "int"), (8, 2_000_003, 130, "int"), (8, 900, 100, "float"),
                                            (8, 5_000_001, 1, "float"), (16, 700_001, 100, "int"), (8, 300_001, 64, "int"),
                                            (16, 200_003, 200, "float")])
def test_a_single_query_spreads_its_candidates_over_four_lists(psc, m, n, k, lut_kind):
    """One query: the three empty slots of the tile hold copies of its tables, every wave feeds the
    list of slot wave % 4 and the four lists are merged when the slice ends (one slice for small
    databases, 256 for large ones).  Exact ties (small-integer tables) must come out in id order."""
    codes, qcodes, lut = _rand_problem(m, n, 1, seed=400 + k, lut_kind=lut_kind)
    nb = 8 * m
    for ht in (nb // 4, nb * 3 // 8, nb // 2 - 3):
        print(f"single query m={m} n={n} k={k} ht={ht}", flush=True)
        got_ids, got_d = _run(psc, lut, qcodes, codes, ht, k)
        ref = O.scan(lut.astype(np.float64), qcodes, codes, ht, k)
        nd = assert_topk_matches(got_ids, got_d, ref, lut.astype(np.float64), qcodes, codes, ht, what=f"single m={m} ht={ht}")
        if lut_kind == "int":
            assert nd == 0


@pytest.mark.parametrize("m", [8, 16])
def test_hamming_filter_is_bit_exact(psc, m):
    codes, qcodes, _ = _rand_problem(m, 20_011, 23, seed=7 + m, lut_kind="int")
    want = O.hamming_matrix(qcodes, codes)
    for ht in (0, 2 * m, 3 * m, 4 * m, 8 * m):
        ns, hd = psc.hamming_filter(_dev(qcodes), _dev(codes), ht, want_distances=True)
        torch.cuda.synchronize()
        assert np.array_equal(hd.cpu().numpy().astype(np.int32), want)
        assert np.array_equal(ns.cpu().numpy(), (want <= ht).sum(axis=1))
        ref = O.scan(np.zeros((23, m, 256)), qcodes, codes, ht, 1)
        assert np.array_equal(ns.cpu().numpy(), ref["nsurv"])


@pytest.mark.parametrize("m", [8, 16])
def test_survivor_set_through_the_fused_scan(psc, m):
    """With k above the number of survivors the result lists exactly the survivor set."""
    codes, qcodes, lut = _rand_problem(m, 60_000, 11, seed=50 + m, lut_kind="float")
    ht = 2 * m + 2
    ref = O.scan(lut.astype(np.float64), qcodes, codes, ht, 1024, want_bitmap=True)
    assert ref["nsurv"].max() < 1024 and ref["nsurv"].max() > 0
    got_ids, got_d = _run(psc, lut, qcodes, codes, ht, 1024)
    for q in range(11):
        surv = np.flatnonzero(ref["bitmap"][q])
        assert sorted(got_ids[q][got_ids[q] >= 0].tolist()) == surv.tolist()


def test_hand_built_patterns_through_the_scan(psc):
    """Row r of the database has exactly r bits set; the query code is zero; table = first byte."""
    for m in (8, 16):
        nb = 8 * m
        codes = np.zeros((nb + 1, m), np.uint8)
        for r in range(nb + 1):
            full, rem = divmod(r, 8)
            codes[r, :full] = 0xFF
            if rem:
                codes[r, full] = (1 << rem) - 1
        lut = np.zeros((1, m, 256), np.float32)
        lut[0, m - 1, :] = 1.0 + np.arange(256)
        qc = np.zeros((1, m), np.uint8)
        for ht in (0, 1, 7, 8, 9, nb // 2, nb - 1, nb):
            got_ids, got_d = _run(psc, lut, qc, codes, ht, nb + 5)
            ref = O.scan(lut.astype(np.float64), qc, codes, ht, nb + 5)
            assert np.array_equal(got_ids, ref["ids"]) and (got_ids[0] >= 0).sum() == ht + 1
            assert np.array_equal(got_d[got_ids >= 0], ref["dists"][ref["ids"] >= 0])


def test_edge_sizes(psc):
    m, k = 8, 5
    lut = np.ones((3, m, 256), np.float32)
    qc = np.zeros((3, m), np.uint8)
    # empty database: all padding
    ids, d = _run(psc, lut, qc, np.zeros((0, m), np.uint8), 64, k)
    assert np.all(ids == -1) and np.all(np.isinf(d))
    # no queries
    ids, d = psc.scan(_dev(lut[:0]), _dev(qc[:0]), _dev(np.zeros((10, m), np.uint8)), 64, k)
    assert ids.shape == (0, k)
    # tiny databases
    for n in (1, 2, 63, 64, 65, 127, 129):
        codes = W.random_codes(n, m, seed=n)
        ids, d = _run(psc, lut, qc, codes, 64, k)
        ref = O.scan(lut.astype(np.float64), qc, codes, 64, k)
        assert np.array_equal(ids, ref["ids"]), n
    # bad arguments are errors, not crashes
    with pytest.raises(psc.PscError):
        psc.scan(_dev(lut), _dev(qc), _dev(W.random_codes(10, m, 1)), 64, 0)
    with pytest.raises(psc.PscError):
        psc.scan(_dev(lut), _dev(qc), _dev(W.random_codes(10, m, 1)), -1, 5)


def test_scan_is_deterministic(psc):
    codes, qcodes, lut = _rand_problem(8, 200_000, 64, seed=9, lut_kind="float")
    a = _run(psc, lut, qcodes, codes, 26, 100)
    b = _run(psc, lut, qcodes, codes, 26, 100)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


@pytest.mark.parametrize("m", [8, 16])
def test_hamming_histogram_is_bit_exact(psc, m):
    """Threshold adjustment (Section 4.2): the pair histogram equals the oracle's, count for count,
    and both sides pick the same threshold for a 95 % filter."""
    codes, qcodes, _ = _rand_problem(m, 300_007, 29, seed=40 + m, lut_kind="int")
    got = psc.hamming_histogram(_dev(qcodes), _dev(codes))
    torch.cuda.synchronize()
    want = O.hamming_histogram(qcodes, codes)
    assert np.array_equal(got.cpu().numpy(), want)
    assert psc.threshold_for_rate(got, 0.05) == O.threshold_for_rate(want, 0.05)
    empty = psc.hamming_histogram(_dev(qcodes), torch.empty((0, m), dtype=torch.uint8, device="cuda"))
    assert int(empty.sum()) == 0
