"""Python face of the CPU oracle -- TEST INFRASTRUCTURE ONLY.

Thin ctypes marshalling over `psc_oracle.c` (all arithmetic of the search path
is in that file, in double precision), plus the two training steps that are
naturally array code: Lloyd k-means for the product quantizer and the loop over
sub-quantizers around the annealing of the index assignment.

Nothing in the product path may import this module.

`kmeans` is pinned on small inputs whose result the mathematics fixes (one centroid, as many
centroids as points, separated pairs from every start, the refill of an empty cluster, the fixed
point checked by brute force).  Parity unpinned: which local minimum k-means reaches on real data
(`train_pq`, `ivf_train_coarse`: it depends on the rows the start draws; objective never rises) and
which local minimum the annealing ends in (`anneal`, `optimize_index_assignment`); see the tests
named test_oracle_*.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

__all__ = [
    "hamming", "hamming_matrix", "hamming_histogram", "threshold_for_rate", "encode", "decode", "build_lut", "query_codes", "scan",
    "search_flat", "ivf_search", "knn_graph", "exact_knn", "recall_at", "train_pq",
    "centroid_distances", "distance_stats", "f_map", "targets_weights", "polyd_loss",
    "swap_delta", "anneal", "apply_assignment", "optimize_index_assignment", "draw_u64",
    "ivf_train_coarse", "ivf_build_lists", "kmeans", "nearest", "num_threads", "rotate",
    "disidx", "neighbour_ranks", "rank_violations", "ell", "polyr_loss", "polyr_swap_delta", "anneal_ranking",
    "optimize_index_assignment_ranking", "search_by_code_distance",
    "imi_train_coarse", "imi_build_lists", "imi_search",
]

_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        _lib.orc_f.restype = C.c_double
        _lib.orc_polyd_loss.restype = C.c_double
        _lib.orc_swap_delta.restype = C.c_double
        _lib.orc_ell.restype = C.c_double
        _lib.orc_polyr_loss.restype = C.c_double
        _lib.orc_polyr_swap_delta.restype = C.c_double
        _lib.orc_draw_u64.restype = C.c_uint64
        _lib.orc_draw_u64.argtypes = [C.c_uint64, C.c_uint64]
    return _lib


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle use (OMP_NUM_THREADS or the core count)."""
    v = os.environ.get("OMP_NUM_THREADS")
    if v:
        try:
            return int(v.split(",")[0])
        except ValueError:
            pass
    return os.cpu_count() or 1


def _p(a, t=C.c_void_p):
    return a.ctypes.data_as(t) if a is not None else None


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _u8(a):
    return np.ascontiguousarray(a, dtype=np.uint8)


# ----------------------------------------------------------------------------- Hamming
def hamming(a, b) -> int:
    a, b = _u8(a).ravel(), _u8(b).ravel()
    assert a.size == b.size
    return int(_L().orc_hamming(_p(a), _p(b), C.c_int(a.size)))


def hamming_matrix(qcodes, codes) -> np.ndarray:
    qcodes, codes = _u8(qcodes), _u8(codes)
    nq, m = qcodes.shape
    n = codes.shape[0]
    out = np.empty((nq, n), dtype=np.int32)
    _L().orc_hamming_matrix(_p(qcodes), C.c_int64(nq), _p(codes), C.c_int64(n), C.c_int(m), _p(out))
    return out


def hamming_histogram(qcodes, codes, chunk: int = 1 << 20) -> np.ndarray:
    """Number of (query code, code) pairs at every Hamming distance 0..8m, int64 [8m+1]: the
    statistic the threshold is adjusted on (Section 4.2, "adjusted on the training sets")."""
    qcodes, codes = _u8(qcodes), _u8(codes)
    nbits = 8 * qcodes.shape[1]
    hist = np.zeros(nbits + 1, dtype=np.int64)
    for s in range(0, codes.shape[0], chunk):
        h = hamming_matrix(qcodes, codes[s:s + chunk])
        hist += np.bincount(h.ravel(), minlength=nbits + 1)
    return hist


def threshold_for_rate(hist, max_keep_fraction: float) -> int:
    """Largest ht such that the filter keeps at most `max_keep_fraction` of the pairs counted in
    `hist` (Section 4.2: the threshold that filters out at least 1 - max_keep_fraction of the
    points); -1 if even ht = 0 keeps more."""
    hist = np.asarray(hist, dtype=np.int64)
    total = int(hist.sum())
    assert total > 0
    ht = -1
    kept = 0
    for h, c in enumerate(hist.tolist()):
        kept += c
        if kept <= max_keep_fraction * total:
            ht = h
        else:
            break
    return ht


# ----------------------------------------------------------------------------- transformation before the quantizer
def rotate(x, r) -> np.ndarray:
    """The linear map applied to every vector before the product quantizer (Section 4.3: an
    optimized rotation before encoding; the additional results also reduce the dimension with it):
    y [n, dout] = x [n, din] . r^T for r [dout, din], in double precision."""
    x, r = _f64(x), _f64(r)
    assert x.shape[1] == r.shape[1]
    return x @ r.T


# ----------------------------------------------------------------------------- PQ codes, tables
def encode(x, codebook) -> np.ndarray:
    """codes [n, m] uint8; codebook [m, 256, dsub]."""
    x, cb = _f64(x), _f64(codebook)
    m, nc, dsub = cb.shape
    assert nc == 256 and x.shape[1] == m * dsub
    codes = np.empty((x.shape[0], m), dtype=np.uint8)
    _L().orc_encode(_p(x), C.c_int64(x.shape[0]), C.c_int(m * dsub), C.c_int(m), _p(cb), _p(codes))
    return codes


def decode(codes, codebook) -> np.ndarray:
    codes, cb = _u8(codes), _f64(codebook)
    m, _, dsub = cb.shape
    x = np.empty((codes.shape[0], m * dsub), dtype=np.float64)
    _L().orc_decode(_p(codes), C.c_int64(codes.shape[0]), C.c_int(m * dsub), C.c_int(m), _p(cb), _p(x))
    return x


def build_lut(queries, codebook) -> np.ndarray:
    """lut [nq, m, 256] float64: squared distance of query sub-vector j to centroid c."""
    q, cb = _f64(queries), _f64(codebook)
    m, _, dsub = cb.shape
    assert q.shape[1] == m * dsub
    lut = np.empty((q.shape[0], m, 256), dtype=np.float64)
    _L().orc_build_lut(_p(q), C.c_int64(q.shape[0]), C.c_int(m * dsub), C.c_int(m), _p(cb), _p(lut))
    return lut


def query_codes(lut) -> np.ndarray:
    lut = _f64(lut)
    nq, m, _ = lut.shape
    qc = np.empty((nq, m), dtype=np.uint8)
    _L().orc_query_codes(_p(lut), C.c_int64(nq), C.c_int(m), _p(qc))
    return qc


# ----------------------------------------------------------------------------- scans
def disidx(a, b) -> int:
    """Number of sub-quantizers whose index differs (Section 3.3, second paragraph)."""
    a, b = _u8(a).ravel(), _u8(b).ravel()
    assert a.size == b.size
    return int(_L().orc_disidx(_p(a), _p(b), C.c_int(a.size)))


FILTERS = {"hamming": 0, "disidx": 1}


def scan(lut, qcodes, codes, ht: int, k: int, ext_ids=None, skip_id=None, want_bitmap=False, filter="hamming"):
    """Filter (keep iff distance <= ht), ADC on survivors, first k by (dist, id).  filter:
    "hamming" = Hamming distance between the codes read as bit strings (the polysemous filter);
    "disidx" = number of differing indexes (the comparison baseline of Section 4.2).

    Returns dict(ids [nq,k] int64, dists [nq,k] float64, nsurv [nq] int64[, bitmap [nq,n] uint8]).
    """
    lut, qcodes, codes = _f64(lut), _u8(qcodes), _u8(codes)
    nq, m, _ = lut.shape
    n = codes.shape[0]
    assert qcodes.shape == (nq, m) and (n == 0 or codes.shape[1] == m)
    ids = np.empty((nq, k), dtype=np.int64)
    dists = np.empty((nq, k), dtype=np.float64)
    nsurv = np.zeros(nq, dtype=np.int64)
    ext = np.ascontiguousarray(ext_ids, dtype=np.int64) if ext_ids is not None else None
    skip = np.ascontiguousarray(skip_id, dtype=np.int64) if skip_id is not None else None
    bitmap = np.zeros((nq, n), dtype=np.uint8) if want_bitmap else None
    if filter == "hamming":
        rc = _L().orc_scan(C.c_int(m), _p(lut), _p(qcodes), C.c_int64(nq), _p(codes), C.c_int64(n),
                           C.c_int(ht), C.c_int(k), _p(ext), _p(skip), _p(ids), _p(dists), _p(nsurv),
                           _p(bitmap))
    else:
        rc = _L().orc_scan_filtered(C.c_int(m), _p(lut), _p(qcodes), C.c_int64(nq), _p(codes), C.c_int64(n),
                                    C.c_int(FILTERS[filter]), C.c_int(ht), C.c_int(k), _p(ext), _p(skip),
                                    _p(ids), _p(dists), _p(nsurv), _p(bitmap))
    if rc != 0:
        raise MemoryError("oracle scan")
    out = dict(ids=ids, dists=dists, nsurv=nsurv)
    if want_bitmap:
        out["bitmap"] = bitmap
    return out


def search_by_code_distance(qcodes, codes, k: int, kind: str = "hamming", chunk: int = 256):
    """The code-only comparison methods of Section 4.2: rank the database by the distance between
    codes alone -- "hamming" = Hamming distance between the codes read as bit strings ("binary"),
    "disidx" = number of differing indexes -- first k by (distance, id).  Returns (ids [nq,k] int64,
    distances [nq,k] int32), padded with -1 when the database is shorter than k."""
    qcodes, codes = _u8(qcodes), _u8(codes)
    nq, n = qcodes.shape[0], codes.shape[0]
    ids = np.full((nq, k), -1, dtype=np.int64)
    dist = np.full((nq, k), -1, dtype=np.int32)
    for s in range(0, nq, chunk):
        qc = qcodes[s:s + chunk]
        if kind == "hamming":
            d = hamming_matrix(qc, codes)
        elif kind == "disidx":
            d = (qc[:, None, :] != codes[None, :, :]).sum(axis=2).astype(np.int32)
        else:
            raise ValueError(kind)
        for q in range(qc.shape[0]):
            order = np.lexsort((np.arange(n), d[q]))[:k]
            ids[s + q, :len(order)] = order
            dist[s + q, :len(order)] = d[q][order]
    return ids, dist


def search_flat(queries, codebook, codes, ht: int, k: int, **kw):
    """Whole flat path: tables from the raw queries, query codes, then `scan`."""
    lut = build_lut(queries, codebook)
    return scan(lut, query_codes(lut), codes, ht, k, **kw)


def ivf_search(queries, codebook, coarse, offsets, codes, list_ids, nprobe: int, ht: int, k: int,
               probed_in=None, qcodes_in=None, want_coarse=False):
    """Inverted-file search with residual codes.  probed_in [nq,nprobe] / qcodes_in
    [nq,nprobe,m] replace the oracle's own coarse ranking / per-list query codes."""
    q, cb, cc = _f64(queries), _f64(codebook), _f64(coarse)
    m, _, dsub = cb.shape
    D = m * dsub
    nlist = cc.shape[0]
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    codes = _u8(codes)
    list_ids = np.ascontiguousarray(list_ids, dtype=np.int32)
    nq = q.shape[0]
    npb = min(nprobe, nlist)
    ids = np.empty((nq, k), dtype=np.int64)
    dists = np.empty((nq, k), dtype=np.float64)
    nsurv = np.zeros(nq, dtype=np.int64)
    probed = np.empty((nq, npb), dtype=np.int32)
    pin = np.ascontiguousarray(probed_in, dtype=np.int32) if probed_in is not None else None
    qin = _u8(qcodes_in) if qcodes_in is not None else None
    if pin is not None:
        assert pin.shape == (nq, npb)
    if qin is not None:
        assert qin.shape == (nq, npb, m)
    cd = np.empty((nq, nlist), dtype=np.float64) if want_coarse else None
    rc = _L().orc_ivf_search(C.c_int(D), C.c_int(m), _p(cb), _p(cc), C.c_int(nlist), _p(offsets),
                             _p(codes), _p(list_ids), _p(q), C.c_int64(nq), C.c_int(nprobe),
                             C.c_int(ht), C.c_int(k), _p(pin), _p(qin), _p(ids), _p(dists), _p(nsurv),
                             _p(probed), _p(cd))
    if rc != 0:
        raise MemoryError("oracle ivf search")
    out = dict(ids=ids, dists=dists, nsurv=nsurv, probed=probed)
    if want_coarse:
        out["coarse_d"] = cd
    return out


def imi_train_coarse(x, k1: int, k2: int, iters: int = 10, seed: int = 0):
    """Product coarse quantizer of the inverted multi-index: one k-means per half of the vectors."""
    x = _f64(x)
    half = x.shape[1] // 2
    return kmeans(x[:, :half], k1, iters, seed)[0], kmeans(x[:, half:], k2, iters, seed + 1)[0]


def imi_build_lists(x, coarse1, coarse2, codebook, base_id: int = 0):
    """Each vector goes to cell (a, b) = nearest centroid of each half (number a * K2 + b); its
    residual to the cell centroid is encoded; vectors are grouped by cell in their original order.
    Returns offsets [K1*K2+1] int64, codes [n, m] uint8, ids [n] int32, cell_no [n] int32."""
    x, c1, c2 = _f64(x), _f64(coarse1), _f64(coarse2)
    half = x.shape[1] // 2
    a, b = nearest(x[:, :half], c1)[0], nearest(x[:, half:], c2)[0]
    cell = (a * c2.shape[0] + b).astype(np.int32)
    res = x - np.concatenate([c1[a], c2[b]], axis=1)
    codes = encode(res, codebook)
    order = np.argsort(cell, kind="stable")
    offsets = np.zeros(c1.shape[0] * c2.shape[0] + 1, dtype=np.int64)
    offsets[1:] = np.cumsum(np.bincount(cell, minlength=c1.shape[0] * c2.shape[0]))
    return offsets, codes[order], (order + base_id).astype(np.int32), cell


def imi_search(queries, codebook, coarse1, coarse2, offsets, codes, list_ids, max_lists: int, max_codes: int,
               ht: int, k: int, cells_in=None, qcodes_in=None):
    """Inverted multi-index search with caps on visited cells and on the codes they hold
    (max_codes <= 0: no cap).  cells_in [nq, max_lists] (padded with -1) / qcodes_in
    [nq, max_lists, m] replace the oracle's own cell order / per-cell bit strings.
    Returns dict(ids, dists, nsurv, cells [nq, max_lists] (-1 padded), ncodes [nq])."""
    q, cb, c1, c2 = _f64(queries), _f64(codebook), _f64(coarse1), _f64(coarse2)
    m, _, dsub = cb.shape
    D = m * dsub
    assert D % 2 == 0 and c1.shape[1] == D // 2 and c2.shape[1] == D // 2 and max_lists >= 1
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    assert offsets.size == c1.shape[0] * c2.shape[0] + 1
    codes = _u8(codes)
    list_ids = np.ascontiguousarray(list_ids, dtype=np.int32)
    nq = q.shape[0]
    ids = np.empty((nq, k), dtype=np.int64)
    dists = np.empty((nq, k), dtype=np.float64)
    nsurv = np.zeros(nq, dtype=np.int64)
    cells = np.empty((nq, max_lists), dtype=np.int32)
    ncodes = np.zeros(nq, dtype=np.int64)
    cin = np.ascontiguousarray(cells_in, dtype=np.int32) if cells_in is not None else None
    qin = _u8(qcodes_in) if qcodes_in is not None else None
    if cin is not None:
        assert cin.shape == (nq, max_lists)
    if qin is not None:
        assert qin.shape == (nq, max_lists, m)
    rc = _L().orc_imi_search(C.c_int(D), C.c_int(m), _p(cb), _p(c1), C.c_int(c1.shape[0]), _p(c2),
                             C.c_int(c2.shape[0]), _p(offsets), _p(codes), _p(list_ids), _p(q), C.c_int64(nq),
                             C.c_int(max_lists), C.c_int64(max_codes), C.c_int(ht), C.c_int(k), _p(cin), _p(qin),
                             _p(ids), _p(dists), _p(nsurv), _p(cells), _p(ncodes))
    if rc != 0:
        raise MemoryError("oracle multi-index search")
    return dict(ids=ids, dists=dists, nsurv=nsurv, cells=cells, ncodes=ncodes)


def knn_graph(x, codebook, codes, ht: int, k: int, rows=None, chunk: int = 1024):
    """k-NN graph mode (Section 5): every database vector in turn is the query; its bit
    string is its own stored code, its tables come from the raw vector, and it is not
    its own neighbour.  `rows` restricts the computation to those row numbers."""
    x = np.asarray(x)
    codes = _u8(codes)
    rows = np.arange(x.shape[0], dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    ids = np.empty((rows.size, k), dtype=np.int64)
    dists = np.empty((rows.size, k), dtype=np.float64)
    nsurv = np.empty(rows.size, dtype=np.int64)
    for s in range(0, rows.size, chunk):
        r = rows[s:s + chunk]
        lut = build_lut(x[r], codebook)
        o = scan(lut, codes[r], codes, ht, k, skip_id=r)
        ids[s:s + r.size], dists[s:s + r.size], nsurv[s:s + r.size] = o["ids"], o["dists"], o["nsurv"]
    return dict(ids=ids, dists=dists, nsurv=nsurv)


def exact_knn(x, queries, k: int, skip_self: bool = False):
    x, q = _f64(x), _f64(queries)
    ids = np.empty((q.shape[0], k), dtype=np.int64)
    dists = np.empty((q.shape[0], k), dtype=np.float64)
    rc = _L().orc_exact_knn(_p(x), C.c_int64(x.shape[0]), _p(q), C.c_int64(q.shape[0]),
                            C.c_int(x.shape[1]), C.c_int(k), C.c_int(int(skip_self)), _p(ids), _p(dists))
    if rc != 0:
        raise MemoryError("oracle exact knn")
    return ids, dists


def recall_at(result_ids, true_nn, R: int) -> float:
    """Fraction of queries whose true nearest neighbour is among the first R results
    (Section 4.1)."""
    result_ids = np.asarray(result_ids)[:, :R]
    true_nn = np.asarray(true_nn).reshape(-1, 1)
    return float((result_ids == true_nn).any(axis=1).mean())


# ----------------------------------------------------------------------------- training
def nearest(x, cent):
    """Index of the nearest centroid (lowest index on ties) and squared distance to it."""
    x, cent = _f64(x), _f64(cent)
    assign = np.empty(x.shape[0], dtype=np.int64)
    dmin = np.empty(x.shape[0], dtype=np.float64)
    _L().orc_nearest(_p(x), C.c_int64(x.shape[0]), C.c_int(x.shape[1]), _p(cent),
                     C.c_int(cent.shape[0]), _p(assign), _p(dmin))
    return assign, dmin


def kmeans(x, ncent: int, iters: int, seed: int, start=None):
    """Lloyd k-means.  Start: the centroids `start` [ncent, d] if given, else `ncent` distinct
    training rows drawn with numpy's default generator seeded by `seed`.  An empty cluster is
    re-seeded with the point of the most populated cluster that lies farthest from that
    cluster's centroid (that cluster's own mean is not recomputed in the same iteration).
    Returns (centroids [ncent, d] float64, objective after each assignment step)."""
    x = _f64(x)
    n, _ = x.shape
    if start is not None:
        cent = _f64(start).copy()
        assert cent.shape == (ncent, x.shape[1])
    else:
        rng = np.random.default_rng(seed)
        cent = x[rng.choice(n, size=ncent, replace=False)].copy()
    objective = []
    for _ in range(iters):
        assign, dmin = nearest(x, cent)
        objective.append(float(dmin.sum()))
        counts = np.bincount(assign, minlength=ncent)
        for c in range(ncent):
            if counts[c] > 0:
                cent[c] = x[assign == c].mean(axis=0)
        for c in np.flatnonzero(counts == 0):
            big = int(counts.argmax())
            members = np.flatnonzero(assign == big)
            far = members[dmin[members].argmax()]
            cent[c] = x[far]
            assign[far] = c
            counts[big] -= 1
            counts[c] += 1
            dmin[far] = 0.0
    return cent, objective


def train_pq(x, m: int, iters: int = 20, seed: int = 0):
    """Product quantizer: one k-means of 256 centroids per sub-space (Section 3, opening).
    Returns codebook [m, 256, dsub] float64."""
    x = _f64(x)
    dsub = x.shape[1] // m
    cb = np.empty((m, 256, dsub), dtype=np.float64)
    for j in range(m):
        cb[j], _ = kmeans(x[:, j * dsub:(j + 1) * dsub], 256, iters, seed + j)
    return cb


def ivf_train_coarse(x, nlist: int, iters: int = 10, seed: int = 0):
    cent, _ = kmeans(x, nlist, iters, seed)
    return cent


def ivf_build_lists(x, coarse, codebook, base_id: int = 0):
    """Assign each vector to its nearest coarse centroid (lowest list on ties), encode the
    residual, group by list keeping the original order inside a list.
    Returns offsets [nlist+1] int64, codes [n, m] uint8, ids [n] int32, list_no [n] int32."""
    x, cc = _f64(x), _f64(coarse)
    nlist = cc.shape[0]
    list_no = nearest(x, cc)[0].astype(np.int32)
    res = x - cc[list_no]
    codes = encode(res, codebook)
    order = np.argsort(list_no, kind="stable")
    counts = np.bincount(list_no, minlength=nlist)
    offsets = np.zeros(nlist + 1, dtype=np.int64)
    offsets[1:] = np.cumsum(counts)
    return offsets, codes[order], (order + base_id).astype(np.int32), list_no


# ----------------------------------------------------------------------------- index assignment
def centroid_distances(cent) -> np.ndarray:
    cent = _f64(cent)
    assert cent.shape[0] == 256
    dmat = np.empty((256, 256), dtype=np.float64)
    _L().orc_centroid_distances(_p(cent), C.c_int(cent.shape[1]), _p(dmat))
    return dmat


def distance_stats(dmat):
    dmat = _f64(dmat)
    mu, sigma = C.c_double(), C.c_double()
    _L().orc_distance_stats(_p(dmat), C.byref(mu), C.byref(sigma))
    return mu.value, sigma.value


def f_map(x: float, mu: float, sigma: float, nbit: int = 8) -> float:
    return float(_L().orc_f(C.c_double(x), C.c_double(mu), C.c_double(sigma), C.c_int(nbit)))


def targets_weights(dmat, mu, sigma, alpha=0.5, nbit=8):
    dmat = _f64(dmat)
    target = np.empty((256, 256), dtype=np.float64)
    weight = np.empty((256, 256), dtype=np.float64)
    _L().orc_targets_weights(_p(dmat), C.c_double(mu), C.c_double(sigma), C.c_double(alpha),
                             C.c_int(nbit), _p(target), _p(weight))
    return target, weight


def polyd_loss(target, weight, pi) -> float:
    return float(_L().orc_polyd_loss(_p(_f64(target)), _p(_f64(weight)), _p(_u8(pi))))


def swap_delta(target, weight, pi, a: int, b: int) -> float:
    return float(_L().orc_swap_delta(_p(_f64(target)), _p(_f64(weight)), _p(_u8(pi)),
                                     C.c_int(a), C.c_int(b)))


def draw_u64(seed: int, c: int) -> int:
    return int(_L().orc_draw_u64(seed, c))


def anneal(cent, n_iter=500_000, t0=0.7, t_decay=0.9 ** (1.0 / 500.0), alpha=0.5, seed=0,
           want_trace=False):
    """Simulated annealing of the index assignment of one sub-quantizer (Section 3.2).
    Returns dict(pi [256] uint8, loss_init, loss_final[, trace])."""
    cent = _f64(cent)
    pi = np.empty(256, dtype=np.uint8)
    li, lf = C.c_double(), C.c_double()
    trace = np.empty(n_iter + 1, dtype=np.float64) if want_trace else None
    _L().orc_anneal(_p(cent), C.c_int(cent.shape[1]), C.c_int64(n_iter), C.c_double(t0),
                    C.c_double(t_decay), C.c_double(alpha), C.c_uint64(seed), _p(pi),
                    C.byref(li), C.byref(lf), _p(trace))
    out = dict(pi=pi, loss_init=li.value, loss_final=lf.value)
    if want_trace:
        out["trace"] = trace
    return out


def apply_assignment(cent, pi) -> np.ndarray:
    cent = _f64(cent)
    out = np.empty_like(cent)
    _L().orc_apply_assignment(_p(cent), C.c_int(cent.shape[1]), _p(_u8(pi)), _p(out))
    return out


def optimize_index_assignment(codebook, n_iter=500_000, t0=0.7, t_decay=0.9 ** (1.0 / 500.0),
                              alpha=0.5, seed=0):
    """Anneal every sub-quantizer independently (seed + j for sub-quantizer j) and renumber
    its centroids.  Returns (new codebook, pis [m,256], (loss_init [m], loss_final [m]))."""
    cb = _f64(codebook)
    m = cb.shape[0]
    out = np.empty_like(cb)
    pis = np.empty((m, 256), dtype=np.uint8)
    li, lf = np.empty(m), np.empty(m)
    for j in range(m):
        r = anneal(cb[j], n_iter, t0, t_decay, alpha, seed + j)
        pis[j], li[j], lf[j] = r["pi"], r["loss_init"], r["loss_final"]
        out[j] = apply_assignment(cb[j], r["pi"])
    return out, pis, (li, lf)


# ----------------------------------------------------------------------------- ranking loss
def neighbour_ranks(dmat) -> np.ndarray:
    """rank[i, j] = place of centroid j among the centroids ordered by distance to i (the nearest
    other centroid has rank 1; rank[i, i] = 0)."""
    dmat = _f64(dmat)
    rank = np.empty((256, 256), dtype=np.int32)
    _L().orc_neighbour_ranks(_p(dmat), _p(rank))
    return rank


def rank_violations(dmat, pi, i: int, j: int) -> int:
    return int(_L().orc_rank_violations(_p(_f64(dmat)), _p(_u8(pi)), C.c_int(i), C.c_int(j)))


def ell(r: int) -> float:
    return float(_L().orc_ell(C.c_int(r)))


def polyr_loss(dmat, rank, pi) -> float:
    rank = np.ascontiguousarray(rank, dtype=np.int32)
    return float(_L().orc_polyr_loss(_p(_f64(dmat)), _p(rank), _p(_u8(pi))))


def polyr_swap_delta(dmat, rank, pi, a: int, b: int) -> float:
    rank = np.ascontiguousarray(rank, dtype=np.int32)
    return float(_L().orc_polyr_swap_delta(_p(_f64(dmat)), _p(rank), _p(_u8(pi)), C.c_int(a), C.c_int(b)))


def anneal_ranking(cent, n_iter=500_000, t0=0.7, t_decay=0.9 ** (1.0 / 500.0), seed=0, want_trace=False):
    """Simulated annealing of one sub-quantizer's index assignment on the ranking loss (Sections
    3.1 and 3.2).  Returns dict(pi [256] uint8, loss_init, loss_final[, trace])."""
    cent = _f64(cent)
    pi = np.empty(256, dtype=np.uint8)
    li, lf = C.c_double(), C.c_double()
    trace = np.empty(n_iter + 1, dtype=np.float64) if want_trace else None
    _L().orc_anneal_ranking(_p(cent), C.c_int(cent.shape[1]), C.c_int64(n_iter), C.c_double(t0),
                            C.c_double(t_decay), C.c_uint64(seed), _p(pi), C.byref(li), C.byref(lf), _p(trace))
    out = dict(pi=pi, loss_init=li.value, loss_final=lf.value)
    if want_trace:
        out["trace"] = trace
    return out


def optimize_index_assignment_ranking(codebook, n_iter=2000, t0=0.7, t_decay=0.9 ** (1.0 / 500.0), seed=0):
    """`optimize_index_assignment` on the ranking loss (slow: an iteration costs milliseconds here)."""
    cb = _f64(codebook)
    m = cb.shape[0]
    out = np.empty_like(cb)
    pis = np.empty((m, 256), dtype=np.uint8)
    li, lf = np.empty(m), np.empty(m)
    for j in range(m):
        r = anneal_ranking(cb[j], n_iter, t0, t_decay, seed + j)
        pis[j], li[j], lf[j] = r["pi"], r["loss_init"], r["loss_final"]
        out[j] = apply_assignment(cb[j], r["pi"])
    return out, pis, (li, lf)
