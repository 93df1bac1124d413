"""Parity of the transformation in front of the quantizer (Section 4.3, additional results) with the
oracle, alone and as the first step of a search (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle as O
import workloads as W
from gpu_util import RTOL, assert_topk_matches

pytestmark = pytest.mark.gpu


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("din,dout,n", [(128, 128, 1000), (128, 64, 513), (96, 80, 300), (256, 128, 129), (1, 8, 5),
                                        (200, 8, 77), (64, 512, 260), (960, 128, 140), (130, 160, 64)])
def test_rotate_matches_oracle(din, dout, n):
    """Sizes that are no multiple of the kernel's tiles (128 rows, 128 output columns, 64 input
    coordinates per step), projections and expansions; entries within float32 accumulation error of
    the double-precision product."""
    import paper_1609_01882_amd as psc
    rng = np.random.default_rng(din * 1000 + dout)
    r = rng.standard_normal((dout, din)).astype(np.float32)
    x = (rng.standard_normal((n, din)) * 50).astype(np.float32)
    idx = psc.Index(dout, 8)
    idx.set_rotation(r)
    y = idx.rotate(_dev(x))
    torch.cuda.synchronize()
    ref = O.rotate(x, r)
    bound = 4e-7 * (np.abs(x.astype(np.float64)) @ np.abs(r.astype(np.float64)).T)   # a few roundings of sum |x_t r_ct|
    err = np.abs(y.cpu().numpy() - ref)
    assert np.all(err <= bound + 1e-30), (err / np.maximum(bound, 1e-30)).max()


def test_rotation_errors_are_reported():
    import paper_1609_01882_amd as psc
    idx = psc.Index(128, 8)
    x = torch.zeros((4, 128), device="cuda")
    with pytest.raises(psc.PscError, match="psc_set_rotation"):
        idx.rotate(x)
    with pytest.raises(psc.PscError):
        idx.set_rotation(np.zeros((128, 5000), np.float32))


@pytest.mark.parametrize("din,m", [(128, 8), (192, 16)])
def test_search_behind_a_rotation_and_reduction(din, m):
    """The whole path with the transformation in front: raw vectors of dimension din are mapped to
    the quantizer's 64 (or 128) dimensions by a random orthonormal projection, encoded, and searched;
    the oracle does the same from the raw vectors in double precision.  Distances to the bar; ids
    equal except on ties and on queries whose bit string falls the other way on a near-tie."""
    import paper_1609_01882_amd as psc
    dout = 64 if m == 8 else 128
    rng = np.random.default_rng(din)
    q_, r_ = np.linalg.qr(rng.standard_normal((din, din)))
    r = (q_ * np.sign(np.diag(r_)))[:dout].astype(np.float32)
    xt = W.sift_like(4000, seed=80, stream=1, dim=din)
    xb = W.sift_like(30_001, seed=80, stream=2, dim=din)
    xq = W.sift_like(40, seed=80, stream=3, dim=din)
    idx = psc.Index(dout, m)
    idx.set_rotation(r)
    idx.train_pq(idx.rotate(_dev(xt)).cpu().numpy(), iters=5, seed=1)
    idx.optimize_index_assignment(n_iter=30_000, seed=2)
    cb = idx.get_codebook()
    yb, yq = idx.rotate(_dev(xb)), idx.rotate(_dev(xq))
    codes = idx.encode(yb)
    ht, k = 3 * m, 20
    ids, d = idx.search(yq, codes, ht, k)
    lut, qc = idx.build_lut(yq)
    torch.cuda.synchronize()
    codes_h, qc = codes.cpu().numpy(), qc.cpu().numpy()
    # the oracle from the raw vectors
    ob, oq = O.rotate(xb, r), O.rotate(xq, r)
    ref_codes = O.encode(ob, cb)
    assert (ref_codes != codes_h).mean() < 1e-3
    lut64 = O.build_lut(oq, cb)
    assert np.allclose(lut.cpu().numpy(), lut64, rtol=1e-4, atol=1e-2)   # (rotated inputs differ by float32 rounding)
    same = np.all(O.query_codes(lut64) == qc, axis=1)
    assert same.mean() > 0.9
    ref = O.scan(lut64, qc, codes_h, ht, k)
    fin = np.isfinite(ref["dists"])
    assert np.array_equal(np.isfinite(d.cpu().numpy()), fin)
    assert np.allclose(d.cpu().numpy()[fin], ref["dists"][fin], rtol=RTOL)
    # and with the library's own tables: the scan contract proper
    lut32 = lut.cpu().numpy().astype(np.float64)
    assert_topk_matches(ids.cpu().numpy(), d.cpu().numpy(), O.scan(lut32, qc, codes_h, ht, k), lut32, qc, codes_h, ht,
                        what=f"rotated search din={din}")
