"""Training left of the scan, on the GPU against the host: k-means of the product quantizer
(Section 3: 256 centroids in each of 8 sub-spaces of 128-D vectors) and of the coarse quantizer of
the inverted file (Section 4.3: 4096 centroids).  One step = one whole training call; the host
legs run fewer iterations (reported per iteration)."""
from __future__ import annotations

import argparse
import json
import time


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=1_000_000, help="training vectors")
    ap.add_argument("--iters", type=int, default=10)
    ap.add_argument("--nlist", type=int, default=4096)
    ap.add_argument("--host-iters", type=int, default=1, help="iterations of the host legs (0: skip them)")
    args = ap.parse_args()
    import torch

    import paper_1609_01882_amd as psc
    import workloads as W
    from ._common import log

    dim, m = 128, 8
    x = W.sift_like_torch(args.n, seed=5, stream=1)
    torch.cuda.synchronize()
    idx = psc.Index(dim, m)

    def wall(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    idx.train_pq_device(x, iters=1, seed=1)  # first launch: code object load, scratch
    t_pq = wall(lambda: idx.train_pq_device(x, iters=args.iters, seed=1))
    idx.ivf_train_coarse_device(x, args.nlist, iters=1, seed=1)
    t_coarse = wall(lambda: idx.ivf_train_coarse_device(x, args.nlist, iters=args.iters, seed=1))
    res = {"workload": "train", "n": args.n, "dim": dim, "m": m, "iters": args.iters,
           "pq_ms_per_iter": round(1e3 * t_pq / args.iters, 3),
           # per row and sub-quantizer 256 x dsub (subtract, multiply-add)
           "pq_tflops": round(3.0 * args.n * 256 * dim / (t_pq / args.iters) / 1e12, 2),
           "nlist": args.nlist, "coarse_ms_per_iter": round(1e3 * t_coarse / args.iters, 3),
           "coarse_tflops": round(2.0 * args.n * args.nlist * dim / (t_coarse / args.iters) / 1e12, 2)}
    if args.host_iters > 0:
        xh = x.cpu().numpy()
        host = psc.Index(dim, m)
        t0 = time.perf_counter()
        host.train_pq(xh, iters=args.host_iters, seed=1)
        res["pq_host_ms_per_iter"] = round(1e3 * (time.perf_counter() - t0) / args.host_iters, 1)
        t0 = time.perf_counter()
        host.ivf_train_coarse(xh, args.nlist, iters=args.host_iters, seed=1)
        res["coarse_host_update_ms_per_iter"] = round(1e3 * (time.perf_counter() - t0) / args.host_iters, 1)
    log(f"[train] {res}")
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
