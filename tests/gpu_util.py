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
