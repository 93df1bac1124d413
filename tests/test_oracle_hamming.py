"""Pins of the oracle's Hamming distance and filter (Section 1; Section 3.3; Section 4.2
"binary" and "dual").  Everything here runs on the CPU."""
import os

import numpy as np
import pytest
from scipy import stats

import oracle as O
import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _patterns():
    out = []
    for line in open(os.path.join(GOLD, "hamming_patterns.txt")):
        line = line.split("#")[0].split()
        if len(line) == 3:
            out.append((bytes.fromhex(line[0]), bytes.fromhex(line[1]), int(line[2])))
    return out


def test_golden_patterns():
    pats = _patterns()
    assert len(pats) >= 16
    for a, b, want in pats:
        a8, b8 = np.frombuffer(a, np.uint8), np.frombuffer(b, np.uint8)
        assert O.hamming(a8, b8) == want
        assert O.hamming(b8, a8) == want


@pytest.mark.parametrize("nbytes", [8, 16])
def test_single_bits_and_prefix_masks(nbytes):
    zero = np.zeros(nbytes, np.uint8)
    for bit in range(8 * nbytes):
        a = zero.copy()
        a[bit // 8] = 1 << (bit % 8)
        assert O.hamming(a, zero) == 1
        # walking prefix: bits 0..bit set -> distance bit+1 from zero
        p = zero.copy()
        full, rem = divmod(bit + 1, 8)
        p[:full] = 0xFF
        if rem:
            p[full] = (1 << rem) - 1
        assert O.hamming(p, zero) == bit + 1
        assert O.hamming(p, a) == bit  # a's bit is inside the prefix


@pytest.mark.parametrize("nbytes", [8, 16])
def test_matrix_against_unpackbits(nbytes):
    # independent route: expand to bits with numpy and count differing positions
    a = W.random_codes(37, nbytes, seed=5)
    b = W.random_codes(211, nbytes, seed=6)
    want = (np.unpackbits(a, axis=1)[:, None, :] != np.unpackbits(b, axis=1)[None, :, :]).sum(axis=2)
    got = O.hamming_matrix(a, b)
    assert got.dtype == np.int32 and np.array_equal(got, want)
    assert got.min() >= 0 and got.max() <= 8 * nbytes  # at most d+1 distinct values (Section 2)


def _zero_lut(nq, m):
    return np.zeros((nq, m, 256))


@pytest.mark.parametrize("m,hts", [(8, (24, 28, 32, 36)), (16, (48, 56, 64, 72))])
def test_filter_rate_follows_binomial(m, hts):
    """Uniformly random codes: the distance to any fixed code is Binomial(8m, 1/2)
    (Section 3.1), so the survivor fraction at threshold ht is its CDF at ht."""
    n, nq = 200_000, 3
    codes = W.random_codes(n, m, seed=21)
    qc = W.random_codes(nq, m, seed=22)
    for ht in hts:
        r = O.scan(_zero_lut(nq, m), qc, codes, ht, 1)
        p = stats.binom.cdf(ht, 8 * m, 0.5)
        sd = np.sqrt(p * (1 - p) / n)
        assert np.all(np.abs(r["nsurv"] / n - p) < 5 * sd + 1e-9), (ht, r["nsurv"] / n, p)


@pytest.mark.parametrize("m", [8, 16])
def test_threshold_is_inclusive_and_nested(m):
    """Keep iff distance <= ht: a code at distance exactly ht survives, at ht+1 it does not;
    survivor sets grow with ht; ht = number of bits keeps everything (pure ADC)."""
    nb = 8 * m
    zero = np.zeros((1, m), np.uint8)
    codes = np.zeros((nb + 1, m), np.uint8)  # row r has exactly r bits set
    for r in range(nb + 1):
        full, rem = divmod(r, 8)
        codes[r, :full] = 0xFF
        if rem:
            codes[r, full] = (1 << rem) - 1
    prev = None
    for ht in range(nb + 1):
        r = O.scan(_zero_lut(1, m), zero, codes, ht, 1, want_bitmap=True)
        bm = r["bitmap"][0].astype(bool)
        assert np.array_equal(bm, np.arange(nb + 1) <= ht)
        assert r["nsurv"][0] == ht + 1
        if prev is not None:
            assert np.all(bm[prev])
        prev = bm
    assert O.scan(_zero_lut(1, m), zero, codes, nb, 1)["nsurv"][0] == nb + 1
    # thresholds above the number of bits behave like the number of bits
    assert O.scan(_zero_lut(1, m), zero, codes, nb + 7, 1)["nsurv"][0] == nb + 1


def test_query_against_its_own_code_is_zero(tiny_pq):
    cb, xb, codes = tiny_pq["cb_poly"], tiny_pq["xb"], tiny_pq["codes"]
    lut = O.build_lut(xb[:20], cb)
    qc = O.query_codes(lut)
    assert np.array_equal(qc, codes[:20])  # the query's bit string is its PQ code
    h = O.hamming_matrix(qc, codes[:20])
    assert np.all(np.diag(h) == 0)


def test_histogram_and_threshold_for_rate():
    """Pins for the threshold adjustment (Section 4.2): the histogram of uniformly random codes
    follows the binomial law; the chosen threshold is the largest one within the allowed rate."""
    from math import comb
    qc = W.random_codes(40, 8, seed=5)
    codes = W.random_codes(50_000, 8, seed=6)
    hist = O.hamming_histogram(qc, codes, chunk=7001)
    assert hist.shape == (65,) and hist.sum() == 40 * 50_000
    # against the matrix, and against the binomial pmf within 6 sigma
    assert np.array_equal(hist, np.bincount(O.hamming_matrix(qc, codes).ravel(), minlength=65))
    tot = hist.sum()
    for h in range(65):
        p = comb(64, h) / 2.0 ** 64
        assert abs(hist[h] - tot * p) <= 6.0 * np.sqrt(tot * p * (1 - p)) + 1.0
    # hand-built histogram: 1, 2, 3, 4 pairs at distances 0..3 (10 in all)
    toy = np.array([1, 2, 3, 4], dtype=np.int64)
    assert O.threshold_for_rate(toy, 0.05) == -1      # even ht = 0 keeps 10 %
    assert O.threshold_for_rate(toy, 0.10) == 0
    assert O.threshold_for_rate(toy, 0.29) == 0
    assert O.threshold_for_rate(toy, 0.30) == 1
    assert O.threshold_for_rate(toy, 0.60) == 2
    assert O.threshold_for_rate(toy, 1.00) == 3
    # binomial law: P[h <= 24] = 3.0 %, P[h <= 25] = 5.2 % for 64 fair bits, so 5 % means ht = 24
    cdf = np.cumsum([comb(64, h) / 2.0 ** 64 for h in range(65)])
    want = int(np.max(np.nonzero(cdf <= 0.05)[0]))
    assert want == 24 and O.threshold_for_rate(hist, 0.05) == want
