"""The entry point that allocates nothing (`psc_scan_static`: the scan's scratch memory is a fixed
array inside the library) against `psc_scan` with a caller's workspace, through the C ABI (needs an
MI355X).  Two calls in a row on the same array, the second with a smaller input: whatever the first
call left behind must not show in the second."""
import numpy as np
import pytest
import torch

import oracle as O
import workloads as W
from gpu_util import assert_topk_matches

pytestmark = pytest.mark.gpu


def _problem(n, nq, seed):
    rng = np.random.default_rng(seed)
    codes = W.random_codes(n, 8, seed=seed)
    qcodes = codes[rng.integers(0, n, size=nq)].copy()
    qcodes[:, 0] ^= rng.integers(0, 256, size=nq).astype(np.uint8)
    lut = (rng.random((nq, 8, 256)) * 1000).astype(np.float32)
    return codes, qcodes, lut


def test_static_scratch_scan_equals_workspace_scan():
    import paper_1609_01882_amd as psc
    cases = [(300_001, 41, 24, 100, 5), (70_003, 9, 22, 10, 6), (2_000_001, 3, 26, 7, 7), (5_000, 1, 64, 20, 8)]
    # the first call on a device looks the array up, at which point the HIP runtime places it in
    # device memory (once per process); from then on the device's free memory must not move
    codes, qcodes, lut = _problem(1000, 1, 4)
    psc.scan_static(*(torch.from_numpy(a).cuda() for a in (lut, qcodes, codes)), 64, 5,
                    (torch.empty((1, 5), dtype=torch.int64, device="cuda"), torch.empty((1, 5), device="cuda")))
    torch.cuda.synchronize()
    for n, nq, ht, k, seed in cases:      # each call is followed by a smaller one or one of another shape
        print(f"static scratch: n={n} nq={nq} ht={ht} k={k}", flush=True)
        codes, qcodes, lut = _problem(n, nq, seed)
        c_dev, q_dev, l_dev = (torch.from_numpy(a).cuda() for a in (codes, qcodes, lut))
        assert psc.scan_workspace_bytes(8, nq, n, k) <= psc.PSC_STATIC_SCRATCH_BYTES
        want_ids, want_d = psc.scan(l_dev, q_dev, c_dev, ht, k)
        out = (torch.full((nq, k), -7, dtype=torch.int64, device="cuda"),
               torch.full((nq, k), -7.0, dtype=torch.float32, device="cuda"))
        free_before = torch.cuda.mem_get_info()[0]
        psc.scan_static(l_dev, q_dev, c_dev, ht, k, out)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before          # the device's free memory did not move
        assert torch.equal(out[0], want_ids) and torch.equal(out[1], want_d)
        ref = O.scan(lut.astype(np.float64), qcodes, codes, ht, k)
        assert_topk_matches(out[0].cpu().numpy(), out[1].cpu().numpy(), ref, lut.astype(np.float64), qcodes, codes, ht,
                            what=f"static n={n}")


def test_static_scratch_scan_rejects_what_does_not_fit():
    import paper_1609_01882_amd as psc
    n, nq, k = 100_000, 40_000, 100     # 40k queries x 100 results: the partial lists alone exceed the array
    assert psc.scan_workspace_bytes(8, nq, n, k) > psc.PSC_STATIC_SCRATCH_BYTES
    z8 = torch.zeros((n, 8), dtype=torch.uint8, device="cuda")
    out = (torch.empty((nq, k), dtype=torch.int64, device="cuda"), torch.empty((nq, k), dtype=torch.float32, device="cuda"))
    with pytest.raises(psc.PscError, match="static array"):
        psc.scan_static(torch.zeros((nq, 8, 256), device="cuda"), torch.zeros((nq, 8), dtype=torch.uint8, device="cuda"),
                        z8, 20, k, out)
