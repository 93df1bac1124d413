"""Inverted-file batch search (Section 4.3): 100M vectors in 4096 lists of residual 64-bit codes,
10k queries, 64 lists probed each, ht=24, k=100.  The database is drawn on the GPU (same recipe as
the host generator) because 100M x 128 floats do not fit in host memory at once.
One step = the whole psc_ivf_search call."""
from __future__ import annotations

import argparse
import json
import os
import time


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--n", type=int, default=0, help="database size (default: the workload's 100M)")
    args = ap.parse_args()
    import torch

    import paper_1609_01882_amd as psc
    import workloads as W
    from ._common import build_ivf_workload, log, time_ms

    cfg = W.get_config("ivf")
    n = args.n or cfg.n_db
    nlist, nprobe, k, ht, nq = cfg.nlist, cfg.nprobe, cfg.k, cfg.hts[0], cfg.n_query
    threads = min(16, os.cpu_count() or 1)
    dev = torch.device("cuda:0")

    idx, offsets, lcodes, lids, counts = build_ivf_workload(psc, cfg, n, dev, threads=threads)

    xq = torch.from_numpy(cfg.vectors("query", n=nq, threads=threads)).to(dev)
    ws = torch.empty(idx.ivf_search_workspace_bytes(nq, nprobe, k), dtype=torch.uint8, device=dev)
    out = (torch.empty((nq, k), dtype=torch.int64, device=dev), torch.empty((nq, k), dtype=torch.float32, device=dev))
    ms = time_ms(lambda: idx.ivf_search(xq, nprobe, ht, k, workspace=ws, out=out), args.steps, args.warmup)
    psc.workspace_status(ws)
    # codes visited: lengths of the probed lists, from a sample of queries
    ns = 64
    _, _, probed, _ = idx.ivf_search(xq[:ns].contiguous(), nprobe, ht, k, want_debug=True)
    torch.cuda.synchronize()
    pairs = float(counts[probed.long()].sum().item()) / ns * nq
    # small batches: latency of one call (the paper's single-query mode, Section 4.3 / Table 2)
    small = []
    for nqs in (1, 16, 256):
        xs = xq[:nqs].contiguous()
        wss = torch.empty(idx.ivf_search_workspace_bytes(nqs, nprobe, k), dtype=torch.uint8, device=dev)
        outs = (torch.empty((nqs, k), dtype=torch.int64, device=dev), torch.empty((nqs, k), dtype=torch.float32, device=dev))
        mss = time_ms(lambda: idx.ivf_search(xs, nprobe, ht, k, workspace=wss, out=outs), 20, 3)
        small.append({"n_query": nqs, "ms_per_call": round(mss, 4), "us_per_query": round(mss * 1e3 / nqs, 2)})
        log(f"[ivf] small batch {small[-1]}")
    res = {"workload": "ivf", "n_db": n, "nlist": nlist, "nprobe": nprobe, "n_query": nq, "k": k, "ht": ht,
           "ms_per_step": round(ms, 3), "us_per_query": ms * 1e3 / nq, "pairs_per_step": pairs,
           "pairs_per_s": pairs / (ms * 1e-3), "workspace_GB": ws.numel() / 1e9, "small_batches": small}
    log(f"[ivf] {res}")
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
