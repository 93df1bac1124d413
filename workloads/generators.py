"""Seeded generators of raw vectors and random codes.

Every stream is defined chunk by chunk: rows [c*CHUNK, (c+1)*CHUNK) of stream
`stream` under seed `seed` are drawn from numpy's default bit generator seeded
with the entropy list [seed, stream, c].  Any slice of a stream can therefore
be regenerated without generating (or holding) the rows before it, and the
result does not depend on how many worker threads produced it.

Two families of vectors:

* `sift_like`: stands in for 128-D SIFT descriptors (the paper's SIFT1M and
  BIGANN sets, Section 4.1): a mixture of `n_centres` isotropic Gaussians whose
  centres are uniform in [0,100]^D, standard deviation 15 per coordinate,
  clipped to [0,255] and rounded to integers, stored as float32.
* `relu_like`: stands in for the 256-D CNN descriptors of the k-NN-graph
  experiment (Section 5): a mixture of `n_centres` Gaussians with N(0,I)
  centres and standard deviation 0.5, negatives set to zero, rows scaled to
  unit L2 norm.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np

CHUNK = 65536

# stream numbers: one per role so that train / database / queries never overlap
STREAM_CENTRES = 0
STREAM_TRAIN = 1
STREAM_DB = 2
STREAM_QUERY = 3
STREAM_CODES = 4


def mixture_centres(seed: int, n_centres: int, dim: int, kind: str = "uniform100") -> np.ndarray:
    """Centres of the Gaussian mixture, float64 [n_centres, dim]."""
    rng = np.random.default_rng([seed, STREAM_CENTRES, 0])
    if kind == "uniform100":
        return rng.uniform(0.0, 100.0, size=(n_centres, dim))
    if kind == "normal":
        return rng.standard_normal(size=(n_centres, dim))
    raise ValueError(kind)


def _chunks(start: int, n: int):
    """Yield (chunk index, first row inside chunk, rows taken, output offset)."""
    out = 0
    row = start
    end = start + n
    while row < end:
        c = row // CHUNK
        lo = row - c * CHUNK
        take = min(CHUNK - lo, end - row)
        yield c, lo, take, out
        out += take
        row += take


def _run(jobs, fn, threads: int):
    if threads <= 1 or len(jobs) <= 1:
        for j in jobs:
            fn(*j)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(lambda j: fn(*j), jobs))


def sift_like(n: int, seed: int, stream: int, start: int = 0, dim: int = 128,
              n_centres: int = 100, sigma: float = 15.0, threads: int = 8,
              out: np.ndarray | None = None) -> np.ndarray:
    """Rows [start, start+n) of a SIFT-like stream, float32 [n, dim]."""
    centres = mixture_centres(seed, n_centres, dim, "uniform100").astype(np.float32)
    if out is None:
        out = np.empty((n, dim), dtype=np.float32)
    assert out.shape == (n, dim) and out.dtype == np.float32

    def fill(c, lo, take, off):
        rng = np.random.default_rng([seed, stream, c])
        comp = rng.integers(0, n_centres, size=CHUNK)
        noise = rng.standard_normal(size=(CHUNK, dim), dtype=np.float32)
        v = centres[comp[lo:lo + take]] + np.float32(sigma) * noise[lo:lo + take]
        np.clip(v, 0.0, 255.0, out=v)
        np.rint(v, out=v)
        out[off:off + take] = v

    _run(list(_chunks(start, n)), fill, threads)
    return out


def relu_like(n: int, seed: int, stream: int, start: int = 0, dim: int = 256,
              n_centres: int = 1000, sigma: float = 0.5, threads: int = 8,
              out: np.ndarray | None = None) -> np.ndarray:
    """Rows [start, start+n) of a ReLU-like unit-norm stream, float32 [n, dim]."""
    centres = mixture_centres(seed, n_centres, dim, "normal").astype(np.float32)
    if out is None:
        out = np.empty((n, dim), dtype=np.float32)
    assert out.shape == (n, dim) and out.dtype == np.float32

    def fill(c, lo, take, off):
        rng = np.random.default_rng([seed, stream, c])
        comp = rng.integers(0, n_centres, size=CHUNK)
        noise = rng.standard_normal(size=(CHUNK, dim), dtype=np.float32)
        v = centres[comp[lo:lo + take]] + np.float32(sigma) * noise[lo:lo + take]
        np.maximum(v, 0.0, out=v)
        nrm = np.sqrt((v.astype(np.float64) ** 2).sum(axis=1))
        nrm[nrm == 0.0] = 1.0
        out[off:off + take] = (v / nrm[:, None]).astype(np.float32)

    _run(list(_chunks(start, n)), fill, threads)
    return out


def sift_like_torch(n: int, seed: int, stream: int, start: int = 0, dim: int = 128, n_centres: int = 100,
                    sigma: float = 15.0, device="cuda"):
    """Same recipe as `sift_like`, drawn on `device` with torch's generator (one generator per
    chunk, seeded from (seed, stream, chunk)); for databases too large to generate on the host.
    The draws differ from the numpy stream of `sift_like`; centres are the same."""
    import torch

    centres = torch.from_numpy(mixture_centres(seed, n_centres, dim, "uniform100").astype(np.float32)).to(device)
    out = torch.empty((n, dim), dtype=torch.float32, device=device)
    for c, lo, take, off in _chunks(start, n):
        g = torch.Generator(device=device)
        g.manual_seed((seed * 1_000_003 + stream) * 1_000_003 + c)
        comp = torch.randint(0, n_centres, (CHUNK,), generator=g, device=device)
        noise = torch.randn((CHUNK, dim), generator=g, device=device, dtype=torch.float32)
        v = centres[comp[lo:lo + take]] + sigma * noise[lo:lo + take]
        out[off:off + take] = v.clamp_(0.0, 255.0).round_()
    return out


def random_codes(n: int, nbytes: int, seed: int, start: int = 0) -> np.ndarray:
    """Uniformly random byte codes, uint8 [n, nbytes] (every bit fair and independent)."""
    out = np.empty((n, nbytes), dtype=np.uint8)
    for c, lo, take, off in _chunks(start, n):
        rng = np.random.default_rng([seed, STREAM_CODES, c, nbytes])
        blk = rng.integers(0, 256, size=(CHUNK, nbytes), dtype=np.uint8)
        out[off:off + take] = blk[lo:lo + take]
    return out


@dataclasses.dataclass(frozen=True)
class WorkloadConfig:
    """Shape of one named workload (the five configurations this build is measured on)."""
    name: str
    family: str          # "sift_like" | "relu_like"
    dim: int
    m: int               # sub-quantizers = bytes per code
    n_train: int
    n_db: int
    n_query: int         # 0 means "every database vector is a query" (graph mode)
    hts: tuple
    k: int
    seed: int
    nlist: int = 0       # >0: IVF with this many coarse lists
    nprobe: int = 0

    def vectors(self, role: str, n: int | None = None, start: int = 0, threads: int = 8,
                out: np.ndarray | None = None) -> np.ndarray:
        stream = {"train": STREAM_TRAIN, "db": STREAM_DB, "query": STREAM_QUERY}[role]
        full = {"train": self.n_train, "db": self.n_db,
                "query": self.n_query if self.n_query else self.n_db}[role]
        if role == "query" and self.n_query == 0:
            stream = STREAM_DB          # graph mode: the queries are the database rows
        if n is None:
            n = full - start
        gen = sift_like if self.family == "sift_like" else relu_like
        return gen(n, self.seed, stream, start=start, dim=self.dim, threads=threads, out=out)


CONFIGS = {
    "tiny": WorkloadConfig("tiny", "sift_like", 128, 8, 10_000, 100_000, 100, (24,), 10, seed=1609),
    "flat64": WorkloadConfig("flat64", "sift_like", 128, 8, 100_000, 10_000_000, 10_000,
                             (16, 20, 24, 28, 32, 64), 100, seed=1882),
    "flat128": WorkloadConfig("flat128", "sift_like", 128, 16, 100_000, 10_000_000, 10_000,
                              (40, 48, 56, 64, 128), 100, seed=1883),
    "ivf": WorkloadConfig("ivf", "sift_like", 128, 8, 100_000, 100_000_000, 10_000, (24,), 100,
                          seed=1884, nlist=4096, nprobe=64),
    "graph": WorkloadConfig("graph", "relu_like", 256, 8, 100_000, 1_000_000, 0, (20,), 10,
                            seed=1885),
}


def get_config(name: str) -> WorkloadConfig:
    return CONFIGS[name]
