"""Flat scan of 10M 128-bit codes by 10k queries, k=100, for every threshold of the workload
(the 16-byte setting of Table 1).  One step = tables + query codes + fused scan + merge."""
from __future__ import annotations

import argparse
import json
import os
import time


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    args = ap.parse_args()
    import torch

    import paper_1609_01882_amd as psc
    import workloads as W
    from ._common import log, time_ms, trained_index

    cfg = W.get_config("flat128")
    threads = min(16, os.cpu_count() or 1)
    dev = torch.device("cuda:0")
    idx = trained_index(psc, cfg, cfg.vectors("train", threads=threads))
    q = torch.from_numpy(cfg.vectors("query", threads=threads)).to(dev)
    codes = torch.empty((cfg.n_db, cfg.m), dtype=torch.uint8, device=dev)
    t0 = time.time()
    for s in range(0, cfg.n_db, 1_000_000):
        c = min(1_000_000, cfg.n_db - s)
        idx.encode(torch.from_numpy(cfg.vectors("db", n=c, start=s, threads=threads)).to(dev), out=codes[s:s + c])
    torch.cuda.synchronize()
    log(f"[setup] database encoded in {time.time() - t0:.1f}s")
    nq, n, k = cfg.n_query, cfg.n_db, cfg.k
    ws = torch.empty(idx.search_workspace_bytes(nq, n, k), dtype=torch.uint8, device=dev)
    out = (torch.empty((nq, k), dtype=torch.int64, device=dev), torch.empty((nq, k), dtype=torch.float32, device=dev))
    rows = []
    for ht in cfg.hts:
        ms = time_ms(lambda: idx.search(q, codes, ht, k, workspace=ws, out=out), args.steps, args.warmup)
        psc.workspace_status(ws)
        surv = psc.hamming_filter(idx.build_lut(q[:256])[1], codes, ht).double().mean().item() / n
        rows.append(dict(ht=ht, ms_per_step=round(ms, 3), pairs_per_s=nq * n / (ms * 1e-3),
                         alu_frac=9 * nq * n / (ms * 1e-3) / (256 * 4 * 16 * 2.4e9), survivor_rate=surv))
        log(f"[flat128] {rows[-1]}")
    print(json.dumps({"workload": "flat128", "n_db": n, "n_query": nq, "k": k, "code_bits": 128,
                      "ops_per_pair": 9, "sweep": rows}), flush=True)


if __name__ == "__main__":
    main()
