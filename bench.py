#!/usr/bin/env python3
"""Benchmark of the polysemous search hot path on one MI355X.

One "step" = one pass of the whole flat search path over the flat 64-bit workload:
ADC tables + query codes for the 10,000-query batch, the fused Hamming-filter + ADC + top-k
scan over the 10,000,000 64-bit codes, and the merge of the partial lists -- with queries,
codebook and codes already resident in HBM.  Inputs are seeded and synthetic (SIFT-like
mixture, see workloads/).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--ht 24] [--small] [--no-sweep] [--no-cpu] [--no-small-batch]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3e12 32-bit integer lane-ops/s
# (half of the 78.6 TFLOP/s non-packed fp32 vector rate, which counts an FMA as two).
PEAK_INT_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# LDS: 128 bytes per clock and compute unit.  The ADC of a survivor gathers m 4-byte table entries.
PEAK_LDS_TBPS = 256 * 128 * 2.4e9 / 1e12
# Algorithmic integer work per (query, code) pair: per 32-bit word one xor and one
# popcount-accumulate, plus one compare against the threshold.
OPS_PER_PAIR = {8: 5, 16: 9}

# Bytes per scan launch between L2 and the memory fabric, measured with rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE (two runs, scaled by what the same counters read for a 1 GiB copy:
# x2.0 and x1.0), see profiles/; keyed by (kernel, ht) on the flat64 workload.
MEASURED_TRAFFIC_BYTES = {("scan_mfma_kernel<16>", 24): 1.9229e10, ("scan_kernel<8,8,8>", 24): 9.7279e10}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--ht", type=int, default=24)
    ap.add_argument("--small", action="store_true", help="1M codes / 1000 queries (quick check)")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-small-batch", action="store_true",
                    help="skip the memory-bound side measurement (1 and 16 queries over 400M codes)")
    ap.add_argument("--cpu-queries", type=int, default=1024)
    ap.add_argument("--filter-route", choices=["auto", "popcount", "mfma"], default="auto",
                    help="which Hamming filter the fused scan uses: the library's own choice (matrix cores "
                         "below about 10%% survivors), or one of the two forced (PSC_FILTER_ROUTE)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (known traffic, for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.filter_route != "auto":
        os.environ["PSC_FILTER_ROUTE"] = args.filter_route
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build measures one GPU only (the path would shard by splitting the query "
            "batch, or the database rows with one k-way merge of the partial lists); run with --gpus 1")
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1609_01882_amd as psc
    import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.backends.cuda.matmul.allow_tf32 = False
    cfg = W.get_config("flat64")
    n_db, nq, k, m = cfg.n_db, cfg.n_query, cfg.k, cfg.m
    if args.small:
        n_db, nq = 1_000_000, 1_000
    threads = min(16, os.cpu_count() or 1)

    # ------------------------------------------------------------------ set-up (untimed)
    t0 = time.time()
    xt = cfg.vectors("train", threads=threads)
    idx = psc.Index(cfg.dim, m)
    idx.train_pq(xt, iters=20, seed=cfg.seed)
    pi, losses = idx.optimize_index_assignment(seed=cfg.seed)   # the paper's annealing constants
    log(f"[setup] PQ trained + index assignment optimised in {time.time() - t0:.1f}s "
        f"(loss {losses[:, 0].mean():.0f} -> {losses[:, 1].mean():.0f})")

    # the paper's rule for the threshold (Section 4.2): the largest ht that filters out at least
    # 95 % of the pairs of the training set (here: 1000 training vectors against all 100k)
    tcodes = idx.encode(torch.from_numpy(xt).to(dev))
    ht_rule = psc.threshold_for_rate(psc.hamming_histogram(tcodes[:1000].contiguous(), tcodes), 0.05)
    log(f"[setup] threshold that removes >= 95 % of the training pairs: ht = {ht_rule}")

    xq = cfg.vectors("query", n=nq, threads=threads)
    q_dev = torch.from_numpy(xq).to(dev)
    qn = (q_dev * q_dev).sum(dim=1)

    # database: generate, encode and compute the exact nearest neighbour chunk by chunk, so the
    # raw vectors never have to be resident all at once
    t0 = time.time()
    codes = torch.empty((n_db, m), dtype=torch.uint8, device=dev)
    best_d = torch.full((nq,), float("inf"), device=dev)
    best_i = torch.full((nq,), -1, dtype=torch.int64, device=dev)
    chunk = 1_000_000
    for s in range(0, n_db, chunk):
        c = min(chunk, n_db - s)
        xb = torch.from_numpy(cfg.vectors("db", n=c, start=s, threads=threads)).to(dev)
        idx.encode(xb, out=codes[s:s + c])
        # exact squared L2 (integer-valued data: exact in float32)
        d = qn[:, None] - 2.0 * (q_dev @ xb.T) + (xb * xb).sum(dim=1)[None, :]
        dmin, imin = d.min(dim=1)
        better = dmin < best_d
        best_d = torch.where(better, dmin, best_d)
        best_i = torch.where(better, imin + s, best_i)
        del xb, d
    torch.cuda.synchronize()
    log(f"[setup] {n_db} vectors generated, encoded, ground truth done in {time.time() - t0:.1f}s")

    ws = torch.empty(idx.search_workspace_bytes(nq, n_db, k), dtype=torch.uint8, device=dev)
    ids = torch.empty((nq, k), dtype=torch.int64, device=dev)
    dists = torch.empty((nq, k), dtype=torch.float32, device=dev)
    scan_ws = torch.empty(psc.scan_workspace_bytes(m, nq, n_db, k), dtype=torch.uint8, device=dev)

    def step(ht, ev=None):
        """The whole path; the scan launch is bracketed by events when `ev` is given."""
        lut, qc = idx.build_lut(q_dev)
        if ev is not None:
            ev[0].record()
        psc.scan(lut, qc, codes, ht, k, workspace=scan_ws, out=(ids, dists))
        if ev is not None:
            ev[1].record()

    def run(ht, steps, warmup):
        for _ in range(warmup):
            step(ht)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(ht, evs[i])
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / steps
        scan_ms = float(np.mean([a.elapsed_time(b) for a, b in evs]))
        psc.workspace_status(scan_ws)
        return wall * 1e3, scan_ms

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ms_step, scan_ms = run(args.ht, args.steps, args.warmup)
    # the tables and query codes alone (part of every step above), for the record
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        idx.build_lut(q_dev)
    e1.record()
    torch.cuda.synchronize()
    lut_ms = e0.elapsed_time(e1) / 5
    pairs = float(nq) * float(n_db)
    recall10 = float((ids[:, :10] == best_i[:, None]).any(dim=1).float().mean())
    nsurv = psc.hamming_filter(idx.build_lut(q_dev[:256])[1], codes, args.ht)
    torch.cuda.synchronize()
    surv_rate = float(nsurv.double().mean()) / n_db
    log(f"[bench] ht={args.ht}: {ms_step:.2f} ms/step, scan {scan_ms:.2f} ms, "
        f"{pairs / ms_step / 1e9:.1f} G pairs/s... recall@10 {recall10:.4f}, survivors {surv_rate:.4%}")

    sweep = []
    if not args.no_sweep:
        for ht in cfg.hts:
            w, sms = run(ht, 2, 1)
            r10 = float((ids[:, :10] == best_i[:, None]).any(dim=1).float().mean())
            r100 = float((ids[:, :100] == best_i[:, None]).any(dim=1).float().mean())
            ns = psc.hamming_filter(idx.build_lut(q_dev[:256])[1], codes, ht)
            torch.cuda.synchronize()
            rate = float(ns.double().mean()) / n_db
            sweep.append(dict(ht=ht, ms_per_step=round(w, 3), scan_ms=round(sms, 3),
                              pairs_per_s=pairs / (w * 1e-3),
                              # the two rooflines of the path: integer ALU for the filter (every pair),
                              # LDS gathers for the ADC (survivors only); whichever is larger binds
                              alu_frac=OPS_PER_PAIR[m] * pairs / (sms * 1e-3) / 1e12 / PEAK_INT_TOPS,
                              lds_frac=rate * pairs * m * 4 / (sms * 1e-3) / 1e12 / PEAK_LDS_TBPS,
                              recall_at_10=r10, recall_at_100=r100, survivor_rate=rate))
            log(f"[sweep] {sweep[-1]}")

    # ------------------------------------------------------------------ side measurement: few queries
    # One pass over a database much larger than the 256 MB last-level cache for 1 and 16 queries:
    # with so little reuse of a code the scan is bound by HBM reads (8 B per code), not by the ALUs.
    # Uniformly random codes and tables; reported beside the headline, never part of `value`.
    small_batch = []
    if not (args.no_small_batch or args.small):
        n_big = 400_000_000
        g = torch.Generator(device=dev)
        g.manual_seed(cfg.seed)
        big = torch.randint(0, 2 ** 31, (n_big * m // 4,), dtype=torch.int32, device=dev,
                            generator=g).view(torch.uint8).view(n_big, m)
        for nqs in (1, 16):
            qcs = torch.randint(0, 256, (nqs, m), dtype=torch.uint8, device=dev, generator=g)
            luts = torch.rand((nqs, m, 256), device=dev, generator=g) * 1000.0
            wss = torch.empty(psc.scan_workspace_bytes(m, nqs, n_big, k), dtype=torch.uint8, device=dev)
            outs = (torch.empty((nqs, k), dtype=torch.int64, device=dev),
                    torch.empty((nqs, k), dtype=torch.float32, device=dev))
            for hts in (0, 20):
                for _ in range(2):
                    psc.scan(luts, qcs, big, hts, k, workspace=wss, out=outs)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for _ in range(5):
                    psc.scan(luts, qcs, big, hts, k, workspace=wss, out=outs)
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / 5
                gbs = n_big * m / (ms * 1e-3) / 1e9
                small_batch.append(dict(n_db=n_big, n_query=nqs, ht=hts, k=k, ms=round(ms, 4),
                                        code_bytes_GBps=round(gbs, 1), frac_of_8TBps=round(gbs / 8000.0, 4),
                                        pairs_per_s=n_big * nqs / (ms * 1e-3)))
                log(f"[small-batch] {small_batch[-1]}")
        del big

    # ------------------------------------------------------------------ CPU baseline: the oracle
    cpu = None
    if not args.no_cpu:
        import oracle as O
        nqc = min(args.cpu_queries, nq)
        lut, qc = idx.build_lut(q_dev[:nqc])
        psc.scan(lut, qc, codes, args.ht, k, out=(ids[:nqc], dists[:nqc]))
        torch.cuda.synchronize()
        lut_h, qc_h, codes_h = lut.cpu().numpy().astype(np.float64), qc.cpu().numpy(), codes.cpu().numpy()
        t0 = time.perf_counter()
        ref = O.scan(lut_h, qc_h, codes_h, args.ht, k)
        dt = time.perf_counter() - t0
        agree = float((ref["ids"] == ids[:nqc].cpu().numpy()).mean())
        cpu = dict(value=nqc * float(n_db) / dt, unit="pairs/s", cores=O.num_threads(), kind="oracle",
                   sample=f"first {nqc} queries x all {n_db} codes, ht={args.ht}, k={k}, {dt:.1f}s",
                   ids_agree_with_gpu=agree)
        log(f"[cpu] oracle: {cpu}")

    ops = OPS_PER_PAIR[m] * pairs
    achieved = ops / (scan_ms * 1e-3) / 1e12
    # the library's rule: matrix-core filter for 64-bit codes below about one survivor in ten pairs
    on_mfma = args.filter_route != "popcount" and m == 8 and (args.ht <= 26 or args.filter_route == "mfma") and args.ht < 31
    kernel = "scan_mfma_kernel<16>" if on_mfma else "scan_kernel<8,8,8>"
    out = {
        "metric": "codes scanned/sec (Hamming filter+ADC, 64-bit codes, 10M DB) + recall@10",
        "value": pairs / (ms_step * 1e-3),
        "unit": "pairs/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_step,
        "lut_ms": lut_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": ("i8 MFMA Hamming test" if on_mfma else "u32 xor/popcount Hamming test") + " + f32 ADC",
        "data": "synthetic",
        "config": {"workload": "flat64" + ("-small" if args.small else ""), "n_db": n_db, "n_query": nq,
                   "code_bits": 8 * m, "ht": args.ht, "k": k},
        "ht_removing_95pct_of_training_pairs": ht_rule,
        "recall_at_10": recall10,
        "survivor_rate": surv_rate,
        # `achieved` counts the algorithmic work of the filter (5 integer operations per 64-bit pair)
        # against the vector-ALU peak, whichever unit executes it; with the test on the matrix
        # cores the same pairs are also 128 int8 operations each against the 5 POP/s MFMA peak.
        "roofline": {"bound": "alu", "kernel": kernel, "achieved": achieved,
                     "peak": PEAK_INT_TOPS, "unit": "TOP/s (int32 lane-ops)", "frac": achieved / PEAK_INT_TOPS,
                     "ops_per_pair": OPS_PER_PAIR[m], "kernel_ms": scan_ms,
                     "traffic": None if args.small else MEASURED_TRAFFIC_BYTES.get((kernel, args.ht)),
                     "mfma_int8_frac": (128.0 * pairs / (scan_ms * 1e-3) / 5.0e15) if on_mfma else None},
        "cpu_baseline": cpu,
        "sweep": sweep,
        "small_batch": small_batch,
        "paper_context": {"adc_evals_per_s_per_core": 222e6, "hamming_evals_per_s_per_core": 1.19e9,
                          "note": "paper's CPU figures for 8-byte codes, one 2.8 GHz core (Fig. 1)"},
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
