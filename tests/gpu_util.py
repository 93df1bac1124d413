"""Helpers for the GPU parity tests: comparison rules between the HIP path and the oracle."""
import numpy as np

RTOL = 1e-5  # ADC distances: float32 sums on the GPU vs float64 in the oracle


def assert_topk_matches(got_ids, got_d, ref, lut64, qcodes, codes, ht, ext_ids=None, what=""):
    """ids identical to the oracle's except where oracle distances tie within RTOL; distances
    within RTOL; padding identical."""
    ref_ids, ref_d = ref["ids"], ref["dists"]
    assert got_ids.shape == ref_ids.shape and got_d.shape == ref_d.shape, what
    pad = ref_ids < 0
    assert np.array_equal(got_ids < 0, pad), f"{what}: padding differs"
    assert np.all(np.isinf(got_d[pad])), what
    assert np.allclose(got_d[~pad], ref_d[~pad], rtol=RTOL, atol=0.0), \
        f"{what}: max rel err {np.max(np.abs(got_d[~pad] - ref_d[~pad]) / np.maximum(ref_d[~pad], 1e-30))}"
    diff = np.argwhere((got_ids != ref_ids) & ~pad)
    if len(diff) == 0:
        return 0
    pos_of = None
    if ext_ids is not None:
        pos_of = {int(v): i for i, v in enumerate(ext_ids)}
    m = codes.shape[1]
    bits_c = None
    for q, r in diff:
        gid = int(got_ids[q, r])
        row = pos_of[gid] if pos_of is not None else gid
        code = codes[row]
        h = int(np.unpackbits(code ^ qcodes[q]).sum())
        assert h <= ht, f"{what}: query {q} returned id {gid} at Hamming distance {h} > {ht}"
        d = float(sum(lut64[q, j, code[j]] for j in range(m)))
        assert abs(d - ref_d[q, r]) <= RTOL * abs(ref_d[q, r]) + 1e-30, \
            f"{what}: query {q} rank {r}: id {gid} (oracle dist {d}) vs oracle id {ref_ids[q, r]} ({ref_d[q, r]})"
    for q in np.unique(diff[:, 0]):
        assert len(set(got_ids[q][~pad[q]].tolist())) == int((~pad[q]).sum()), f"{what}: duplicate ids"
    return len(diff)


def assert_ivf_topk_matches(got_ids, got_d, ref, xq, cb, coarse, offsets, lcodes, lids, probed, qcodes, ht,
                            build_lut, what=""):
    """Inverted-file results against the oracle run on the same decisions (`probed` [nq][nprobe],
    `qcodes` [nq][nprobe][m]): padding identical, distances within RTOL, ids identical except where
    the oracle's distances tie within RTOL -- and every differing id is re-derived from the index:
    its row lies in one of the query's probed lists, its Hamming distance under that list's bit
    string is within the threshold, and its residual ADC distance (float64 tables built by
    `build_lut` = the oracle's) is the oracle's distance at that rank.  No id repeats in a row."""
    ref_ids, ref_d = ref["ids"], ref["dists"]
    assert got_ids.shape == ref_ids.shape and got_d.shape == ref_d.shape, what
    pad = ref_ids < 0
    assert np.array_equal(got_ids < 0, pad), f"{what}: padding differs"
    assert np.all(np.isinf(got_d[pad])), what
    assert np.allclose(got_d[~pad], ref_d[~pad], rtol=RTOL, atol=0.0), \
        f"{what}: max rel err {np.max(np.abs(got_d[~pad] - ref_d[~pad]) / np.maximum(ref_d[~pad], 1e-30))}"
    for q in range(got_ids.shape[0]):
        row = got_ids[q][~pad[q]]
        assert len(np.unique(row)) == len(row), f"{what}: query {q} returns an id twice"
    diff = np.argwhere((got_ids != ref_ids) & ~pad)
    if len(diff) == 0:
        return 0
    m = lcodes.shape[1]
    for q, r in diff:
        gid = int(got_ids[q, r])
        rows = np.flatnonzero(lids == gid)
        assert len(rows) == 1, f"{what}: query {q} returned id {gid}, stored {len(rows)} times"
        row = int(rows[0])
        lst = int(np.searchsorted(offsets, row, side="right") - 1)
        where = np.flatnonzero(probed[q] == lst)
        assert len(where) == 1, f"{what}: query {q} returned id {gid} of list {lst}, which it did not probe"
        p = int(where[0])
        code = lcodes[row]
        h = int(np.unpackbits(code ^ qcodes[q, p]).sum())
        assert h <= ht, f"{what}: query {q} returned id {gid} at Hamming distance {h} > {ht}"
        lut = build_lut((xq[q].astype(np.float64) - coarse[lst].astype(np.float64))[None, :], cb)[0]
        d = float(sum(lut[j, code[j]] for j in range(m)))
        assert abs(d - ref_d[q, r]) <= RTOL * abs(ref_d[q, r]) + 1e-30, \
            f"{what}: query {q} rank {r}: id {gid} (oracle dist {d}) vs oracle id {ref_ids[q, r]} ({ref_d[q, r]})"
    return len(diff)
