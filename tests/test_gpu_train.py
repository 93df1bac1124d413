"""k-means on the GPU (product quantizer of Section 3, coarse quantizer of Section 4.3) against the
oracle's Lloyd iteration and the library's own host training (needs an MI355X).

An iteration is compared from a common start.  Which cell a row with two nearly equidistant
centroids goes to is decided in the kernel's float32 on both sides: the test takes that decision
from the library's own assignment entry points, checks it against the oracle's distances, and
then checks every new centroid."""
import numpy as np
import pytest
import torch

import oracle as O
import workloads as W

pytestmark = pytest.mark.gpu

CENT_RTOL = 1e-5   # float32 partial sums of a few members, double totals, one rounding to float32
GAP_PQ = 1e-5      # how far (relative) the GPU's cell may be from the nearest one in float64:
GAP_COARSE = 1e-4  # direct float32 differences (PQ) / norms and dot products on the matrix cores (coarse)


@pytest.fixture(scope="module")
def psc():
    import paper_1609_01882_amd as p
    return p


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def start_rows(n, ncent, seed):
    """The documented start: partial Fisher-Yates on the row numbers with SplitMix64 draws."""
    perm = np.arange(n, dtype=np.int64)
    for c in range(ncent):
        r = c + O.draw_u64(seed, c) % (n - c)
        perm[c], perm[r] = perm[r], perm[c]
    return perm[:ncent].copy()


def check_update(x, start, assign, got, ref, gap, what):
    """One Lloyd iteration from `start`.  `assign` = the cells the GPU's own assignment kernel
    gives for `start` (the decision is taken in the kernel's precision on both sides):
    every one of them must be a nearest centroid by the oracle's distances up to `gap`; the new
    centroids must be the means of exactly those members (all cells); and wherever the oracle's
    float64 assignment fills a cell with the same members, its centroid must agree too."""
    x = x.astype(np.float64)
    start = start.astype(np.float64)
    oa, dmin = O.nearest(x, start)
    d_assigned = ((x - start[assign]) ** 2).sum(axis=1)
    assert np.all(d_assigned <= dmin * (1 + gap) + 1e-9), f"{what}: a row went to a cell that is not its nearest"
    scale = np.abs(ref).max()
    ncent = start.shape[0]
    counts = np.bincount(assign, minlength=ncent)
    assert counts.min() > 0, f"{what}: this check is for iterations without empty cells"
    want = np.zeros_like(start)
    np.add.at(want, assign, x)
    want /= counts[:, None]
    err = np.abs(got - want).max()
    assert err <= CENT_RTOL * scale, f"{what}: centroid error {err} (scale {scale})"
    moved = np.zeros(ncent, dtype=bool)
    moved[assign[assign != oa]] = True
    moved[oa[assign != oa]] = True
    assert (~moved).any()
    err = np.abs(got[~moved] - ref[~moved]).max()
    assert err <= CENT_RTOL * scale, f"{what}: centroid error against the oracle {err} (scale {scale})"
    return int(moved.sum())


@pytest.mark.parametrize("dim,m", [(128, 8), (128, 16), (96, 8), (64, 16)])
def test_pq_lloyd_iterations_from_a_common_start(psc, dim, m):
    n, dsub = 20_000, dim // m
    x = W.sift_like(n, seed=31, stream=1)[:, :dim].copy()
    xd = _dev(x)
    idx = psc.Index(dim, m)
    rng = np.random.default_rng(4)
    cb = np.stack([x[rng.choice(n, 256, replace=False), j * dsub:(j + 1) * dsub] for j in range(m)]).astype(np.float32)
    for it in range(3):
        idx.set_codebook(cb)
        cells = idx.encode(xd).cpu().numpy()
        obj = idx.train_pq_device(xd, iters=1, from_current=True)
        got = idx.get_codebook()
        nxt = np.empty_like(cb)
        nmoved = 0
        for j in range(m):
            sub = x[:, j * dsub:(j + 1) * dsub]
            ref, robj = O.kmeans(sub, 256, 1, seed=0, start=cb[j])
            assert np.isclose(obj[0, j], robj[0], rtol=1e-6), (it, j, obj[0, j], robj[0])
            nmoved += check_update(sub, cb[j], cells[:, j].astype(np.int64), got[j], ref, GAP_PQ,
                                   f"iteration {it}, sub-quantizer {j}")
            nxt[j] = ref.astype(np.float32)
        assert nmoved <= 0.02 * m * 256
        cb = nxt  # both sides go on from the oracle's centroids


def test_pq_seeded_start_and_the_host_training(psc):
    """Seeded start: iteration 1 equals the oracle's from the documented starting rows; over
    several iterations the objective never rises and the result quantizes as well as the host
    training from the same seed (the two may part ways at an ambiguous point)."""
    n, dim, m, dsub = 12_000, 128, 8, 16
    x = W.sift_like(n, seed=32, stream=1)
    xd = _dev(x)
    idx = psc.Index(dim, m)
    starts = np.stack([x[start_rows(n, 256, 90 + j), j * dsub:(j + 1) * dsub] for j in range(m)])
    idx.set_codebook(starts)
    cells = idx.encode(xd).cpu().numpy()
    obj1 = idx.train_pq_device(xd, iters=1, seed=90)
    got = idx.get_codebook()
    for j in range(m):
        sub = x[:, j * dsub:(j + 1) * dsub]
        ref, robj = O.kmeans(sub, 256, 1, seed=0, start=starts[j])
        assert np.isclose(obj1[0, j], robj[0], rtol=1e-6)
        check_update(sub, starts[j], cells[:, j].astype(np.int64), got[j], ref, GAP_PQ, f"sub-quantizer {j}")
    obj = idx.train_pq_device(xd, iters=8, seed=90)
    assert np.allclose(obj[0], obj1[0], rtol=1e-9)
    assert np.all(np.diff(obj, axis=0) <= 1e-6 * obj[0])
    cb_dev = idx.get_codebook().astype(np.float64)
    host = psc.Index(dim, m)
    host.train_pq(x, iters=8, seed=90)
    cb_host = host.get_codebook().astype(np.float64)
    xe = W.sift_like(3000, seed=32, stream=2)

    def err(c):
        return ((xe - O.decode(O.encode(xe, c), c)) ** 2).sum(axis=1).mean()
    assert abs(err(cb_dev) - err(cb_host)) < 0.01 * err(cb_host)
    same = np.isclose(cb_dev, cb_host, rtol=0, atol=1e-4 * np.abs(cb_host).max()).all(axis=2).mean()
    assert same > 0.9, same


def test_pq_refill_of_empty_cells(psc):
    """Fewer distinct points than centroids: every iteration has empty cells.  Integer coordinates
    make every distance exact in float32, so the GPU must follow the oracle's rule to the letter
    (farthest member of the most populated cell, lowest row on ties, donor's mean untouched)."""
    rng = np.random.default_rng(8)
    base = rng.integers(0, 40, size=(150, 64)).astype(np.float32)
    x = base[rng.integers(0, 150, size=700)]
    x[:256] = base[rng.integers(0, 150, size=256)]
    xd = _dev(x)
    idx = psc.Index(64, 8)
    cb = np.stack([x[:256, j * 8:(j + 1) * 8] for j in range(8)]).astype(np.float32)  # duplicates among the start
    idx.set_codebook(cb)
    for it in range(3):
        obj = idx.train_pq_device(xd, iters=1, from_current=True)
        got = idx.get_codebook()
        for j in range(8):
            ref, robj = O.kmeans(x[:, j * 8:(j + 1) * 8], 256, 1, seed=0, start=cb[j])
            assert np.isclose(obj[0, j], robj[0], rtol=1e-6)
            assert np.allclose(got[j], ref, rtol=0, atol=1e-5), (it, j, np.abs(got[j] - ref).max())
        cb = got
    # as many distinct rows as centroids, seeded start: the codebook is the set of points
    pts = rng.permutation(256 * 64).astype(np.float32).reshape(256, 64)
    idx.train_pq_device(_dev(pts), iters=2, seed=5)
    got = idx.get_codebook()
    for j in range(8):
        assert sorted(map(tuple, got[j])) == sorted(map(tuple, pts[:, j * 8:(j + 1) * 8]))


def test_pq_longest_sub_vectors(psc):
    """64 coordinates per sub-quantizer: the step kernel's 129 KB of LDS (codebook + private sums)."""
    n, dim, m = 3000, 512, 8
    x = np.random.default_rng(3).normal(size=(n, dim)).astype(np.float32) * 20
    xd = _dev(x)
    idx = psc.Index(dim, m)
    starts = np.stack([x[start_rows(n, 256, 7 + j), j * 64:(j + 1) * 64] for j in range(m)])
    idx.set_codebook(starts)
    cells = idx.encode(xd).cpu().numpy()
    obj = idx.train_pq_device(xd, iters=1, seed=7)
    got = idx.get_codebook()
    for j in range(m):
        sub = x[:, j * 64:(j + 1) * 64]
        ref, robj = O.kmeans(sub, 256, 1, seed=0, start=starts[j])
        assert np.isclose(obj[0, j], robj[0], rtol=1e-6)
        check_update(sub, starts[j], cells[:, j].astype(np.int64), got[j], ref, GAP_PQ, f"sub-quantizer {j}")


@pytest.mark.parametrize("dim,nlist", [(128, 300), (64, 1000), (96, 37), (40, 50)])
def test_coarse_training_on_the_device(psc, dim, nlist):
    """One iteration from the documented seeded start against the oracle; several iterations
    against the host training of the same seed."""
    n = 15_000
    x = np.ascontiguousarray(W.sift_like(n, seed=33, stream=1)[:, :dim])
    xd = _dev(x)
    idx = psc.Index(dim, 8)
    start = x[start_rows(n, nlist, 17)]
    idx.ivf_set_coarse(start)
    cells, _ = idx.ivf_assign_encode(xd, want_codes=False)
    idx.ivf_train_coarse_device(xd, nlist, iters=1, seed=17)
    got = idx.ivf_get_coarse()
    ref, _ = O.kmeans(x, nlist, 1, seed=0, start=start)
    check_update(x, start, cells.cpu().numpy().astype(np.int64), got, ref, GAP_COARSE, f"coarse {dim}/{nlist}")
    idx.ivf_train_coarse_device(xd, nlist, iters=5, seed=17)
    dev = idx.ivf_get_coarse().astype(np.float64)
    host = psc.Index(dim, 8)
    host.ivf_train_coarse(x, nlist, iters=5, seed=17)
    hst = host.ivf_get_coarse().astype(np.float64)
    same = np.isclose(dev, hst, rtol=0, atol=1e-4 * np.abs(hst).max()).all(axis=1).mean()
    assert same > 0.9, same
    _, d_dev = O.nearest(x, dev)
    _, d_hst = O.nearest(x, hst)
    assert abs(d_dev.sum() - d_hst.sum()) < 0.01 * d_hst.sum()


def test_coarse_refill_and_argument_errors(psc):
    rng = np.random.default_rng(9)
    base = rng.integers(0, 30, size=(20, 32)).astype(np.float32)
    x = base[rng.integers(0, 20, size=500)]
    idx = psc.Index(32, 8)
    idx.ivf_train_coarse_device(_dev(x), 64, iters=3, seed=1)  # 20 distinct points, 64 cells
    cent = idx.ivf_get_coarse()
    assert np.isfinite(cent).all()
    host = psc.Index(32, 8)
    host.ivf_train_coarse(x, 64, iters=3, seed=1)  # same start, same assignment kernel, same refill rule
    assert np.allclose(cent, host.ivf_get_coarse(), rtol=0, atol=1e-5)
    with pytest.raises(psc.PscError):
        idx.ivf_train_coarse_device(_dev(x[:10]), 64, iters=1, seed=1)  # fewer rows than cells
    with pytest.raises(psc.PscError):
        psc.Index(128, 8).train_pq_device(_dev(np.zeros((100, 128), np.float32)), iters=1)  # fewer than 256 rows
    with pytest.raises(psc.PscError):
        psc.Index(128, 8).train_pq_device(_dev(np.zeros((300, 128), np.float32)), iters=1, from_current=True)
