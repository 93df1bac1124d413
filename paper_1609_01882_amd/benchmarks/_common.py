"""Shared plumbing of the timing scripts: logging to stderr, event timing, index training."""
from __future__ import annotations

import sys
import time


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_ms(fn, steps, warmup):
    """Mean milliseconds of fn() over `steps` calls after `warmup` untimed ones (events on the
    current stream, which is the stream the library launches on)."""
    import torch

    for _ in range(warmup):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def trained_index(psc, cfg, train_rows, threads=16):
    """Product quantizer trained on `train_rows` with the index assignment optimised
    (the paper's annealing constants, Section 3.2)."""
    t0 = time.time()
    idx = psc.Index(cfg.dim, cfg.m)
    idx.train_pq(train_rows, iters=20, seed=cfg.seed)
    idx.optimize_index_assignment(seed=cfg.seed)
    log(f"[setup] PQ + index assignment in {time.time() - t0:.1f}s")
    return idx


def graph_replay_ms(fn, steps, warmup=3):
    """Mean milliseconds of one replay of fn() recorded into a HIP graph (fn must allocate nothing:
    workspace and outputs handed in), or None when the recording fails.  The recorded call has run
    eagerly before, so whatever happens once per process is done."""
    import torch

    try:
        fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return time_ms(g.replay, steps, warmup)
    except Exception as exc:  # noqa: BLE001  (a figure less, not a failed benchmark)
        log(f"[graph replay] not recorded: {exc}")
        return None


def encode_database(idx, cfg, n, dev, chunk=1_000_000, threads=16):
    """Codes [n][m] of the workload's database stream, generated and encoded chunk by chunk so the
    raw vectors are never resident all at once."""
    import torch

    codes = torch.empty((n, cfg.m), dtype=torch.uint8, device=dev)
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        idx.encode(torch.from_numpy(cfg.vectors("db", n=c, start=s, threads=threads)).to(dev), out=codes[s:s + c])
    return codes


def build_ivf_workload(psc, cfg, n, dev, coarse_train=500_000, coarse_iters=10, pq_train=None, pq_iters=20,
                       sa_iters=500_000, threads=16, chunk=4_000_000):
    """The inverted-file workload (Section 4.3): coarse quantizer, product quantizer of the
    residuals with optimised index assignment, and the n database vectors -- drawn on the GPU --
    assigned, encoded and grouped into lists.  Returns (index, offsets, list codes, list ids, list
    sizes); the index borrows the three tensors."""
    import torch

    import workloads as W

    t0 = time.time()
    idx = psc.Index(cfg.dim, cfg.m)
    idx.ivf_train_coarse(W.sift_like(coarse_train, cfg.seed, 7, threads=threads), cfg.nlist, iters=coarse_iters,
                         seed=cfg.seed)
    coarse = idx.ivf_get_coarse()
    xt = cfg.vectors("train", n=pq_train, threads=threads)
    lt, _ = idx.ivf_assign_encode(torch.from_numpy(xt).to(dev), want_codes=False)
    idx.train_pq(xt - coarse[lt.cpu().numpy()], iters=pq_iters, seed=cfg.seed)   # PQ of the residuals
    idx.optimize_index_assignment(n_iter=sa_iters, seed=cfg.seed)
    log(f"[setup] coarse quantizer, residual PQ, index assignment in {time.time() - t0:.1f}s")
    t0 = time.time()
    list_no = torch.empty(n, dtype=torch.int32, device=dev)
    codes = torch.empty((n, cfg.m), dtype=torch.uint8, device=dev)
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        ln, cd = idx.ivf_assign_encode(W.sift_like_torch(c, cfg.seed, 2, start=s, device=dev))
        list_no[s:s + c] = ln
        codes[s:s + c] = cd
    order = torch.sort(list_no.to(torch.int64), stable=True).indices
    counts = torch.bincount(list_no.to(torch.int64), minlength=cfg.nlist)
    offsets = torch.zeros(cfg.nlist + 1, dtype=torch.int64, device=dev)
    offsets[1:] = torch.cumsum(counts, 0)
    lcodes, lids = codes[order].contiguous(), order.to(torch.int32).contiguous()
    del codes, order, list_no
    idx.ivf_set_lists(offsets, lcodes, lids)
    torch.cuda.synchronize()
    log(f"[setup] {n} vectors assigned, encoded and grouped into lists in {time.time() - t0:.1f}s "
        f"(list sizes {counts.min().item()} / {counts.float().mean().item():.0f} / {counts.max().item()})")
    return idx, offsets, lcodes, lids, counts


def build_imi_workload(psc, cfg, n, k_half, dev, coarse_train=500_000, coarse_iters=10, pq_train=None, pq_iters=20,
                       sa_iters=500_000, threads=16, chunk=4_000_000):
    """The inverted multi-index over the inverted-file workload's vectors (Section 4.3, Table 2):
    product coarse quantizer of k_half x k_half cells (each half trained as a plain coarse quantizer in
    dimension dim/2, on the device), product quantizer of the residuals with optimised index
    assignment, the n database vectors -- drawn on the GPU -- assigned, encoded and grouped by cell.
    Returns (index, offsets, cell codes, cell ids, training residual codes)."""
    import numpy as np
    import torch

    import workloads as W

    t0 = time.time()
    half = cfg.dim // 2
    xc = torch.from_numpy(W.sift_like(coarse_train, cfg.seed, 7, threads=threads)).to(dev)
    cents = []
    for h in range(2):
        tmp = psc.Index(half, 8)
        tmp.ivf_train_coarse_device(xc[:, h * half:(h + 1) * half].contiguous(), k_half, iters=coarse_iters, seed=cfg.seed + h)
        cents.append(tmp.ivf_get_coarse())
    del xc
    idx = psc.Index(cfg.dim, cfg.m)
    idx.imi_set_coarse(cents[0], cents[1])
    xt = cfg.vectors("train", n=pq_train, threads=threads)
    ct = idx.imi_assign_encode(torch.from_numpy(xt).to(dev), want_codes=False)[0].cpu().numpy()
    idx.train_pq(xt - np.concatenate([cents[0][ct // k_half], cents[1][ct % k_half]], axis=1), iters=pq_iters, seed=cfg.seed)
    idx.optimize_index_assignment(n_iter=sa_iters, seed=cfg.seed)
    tcodes = idx.imi_assign_encode(torch.from_numpy(xt).to(dev))[1]
    log(f"[setup] product coarse quantizer {k_half} x {k_half}, residual PQ, index assignment in {time.time() - t0:.1f}s")
    t0 = time.time()
    cell = torch.empty(n, dtype=torch.int32, device=dev)
    codes = torch.empty((n, cfg.m), dtype=torch.uint8, device=dev)
    ws = torch.empty(idx.imi_assign_workspace_bytes(chunk), dtype=torch.uint8, device=dev)
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        ce, cd = idx.imi_assign_encode(W.sift_like_torch(c, cfg.seed, 2, start=s, device=dev), workspace=ws)
        cell[s:s + c] = ce
        codes[s:s + c] = cd
    del ws
    ncell = k_half * k_half
    order = torch.sort(cell.to(torch.int64), stable=True).indices
    offsets = torch.zeros(ncell + 1, dtype=torch.int64, device=dev)
    offsets[1:] = torch.cumsum(torch.bincount(cell.to(torch.int64), minlength=ncell), 0)
    lcodes, lids = codes[order].contiguous(), order.to(torch.int32).contiguous()
    del codes, order, cell
    idx.imi_set_lists(offsets, lcodes, lids)
    torch.cuda.synchronize()
    sizes = offsets[1:] - offsets[:-1]
    log(f"[setup] {n} vectors assigned to {ncell} cells, encoded and grouped in {time.time() - t0:.1f}s "
        f"(codes per cell: mean {n / ncell:.1f}, max {sizes.max().item()}, empty {(sizes == 0).float().mean().item():.1%})")
    return idx, offsets, lcodes, lids, tcodes
