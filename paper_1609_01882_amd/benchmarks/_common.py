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
