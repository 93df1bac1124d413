"""The scan under HIP graph capture (needs an MI355X): `psc_scan_static` allocates nothing and
needs no workspace, so a caller can record it once and replay it.  Every replay -- with new
inputs written into the recorded buffers and eager work of the same library between the replays --
must equal the eager result on the same inputs."""
import numpy as np
import pytest
import torch

import oracle as O
import workloads as W
from gpu_util import assert_topk_matches

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,nq,ht,k", [(300_001, 12, 24, 100), (1_200_003, 1, 22, 10)])
def test_replays_of_a_recorded_scan_equal_eager_calls(n, nq, ht, k):
    import paper_1609_01882_amd as psc
    m = 8
    rng = np.random.default_rng(31 + nq)
    codes = W.random_codes(n, m, seed=61)
    c_dev = torch.from_numpy(codes).cuda()

    def inputs(seed):
        r = np.random.default_rng(seed)
        qc = codes[r.integers(0, n, size=nq)].copy()
        qc[:, 1] ^= r.integers(0, 16, size=nq).astype(np.uint8)
        return (r.random((nq, m, 256)) * 1000).astype(np.float32), qc

    lut_h, qc_h = inputs(1)
    lut_s, qc_s = torch.from_numpy(lut_h).cuda(), torch.from_numpy(qc_h).cuda()      # the recorded buffers
    out_s = (torch.empty((nq, k), dtype=torch.int64, device="cuda"), torch.empty((nq, k), dtype=torch.float32, device="cuda"))
    # everything that happens once per process or per kernel (placing the static array, kernel
    # attributes) happens in an eager call of the same shape, before the recording
    psc.scan_static(lut_s, qc_s, c_dev, ht, k, out_s)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        psc.scan_static(lut_s, qc_s, c_dev, ht, k, out_s)
    for turn in range(4):
        lut_h, qc_h = inputs(100 + turn)
        lut_s.copy_(torch.from_numpy(lut_h))
        qc_s.copy_(torch.from_numpy(qc_h))
        out_s[0].fill_(-7)
        out_s[1].fill_(-7.0)
        print(f"replay {turn}: n={n} nq={nq}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        got_ids, got_d = out_s[0].clone(), out_s[1].clone()
        # eager work of the library between the replays: the same scan with a workspace of its own
        want_ids, want_d = psc.scan(lut_s, qc_s, c_dev, ht, k)
        torch.cuda.synchronize()
        assert torch.equal(got_ids, want_ids) and torch.equal(got_d, want_d), turn
        if turn == 3:
            ref = O.scan(lut_h.astype(np.float64), qc_h, codes, ht, k)
            assert_topk_matches(got_ids.cpu().numpy(), got_d.cpu().numpy(), ref, lut_h.astype(np.float64), qc_h, codes, ht,
                                what=f"replayed scan n={n} nq={nq}")
