"""Thin Python binding of libpsc.so: argument marshalling only.

Every step of the search path runs in the library's HIP kernels; torch is used for device
memory (tensors) and the current stream.  If the shared library is missing this module raises
at import of the first call -- there is no CPU or eager fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("PSC_LIB_PATH") or os.path.join(_HERE, "libpsc.so")
_lib = None

PSC_MAX_K = 1024
PSC_START_SEEDED, PSC_START_CURRENT = 0, 1


class PscError(RuntimeError):
    pass


def lib_path() -> str:
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise PscError(f"{_LIB_PATH} not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = C.CDLL(_LIB_PATH)
    vp, i64, i32, u64, dbl, sz = C.c_void_p, C.c_int64, C.c_int, C.c_uint64, C.c_double, C.c_size_t
    sigs = {
        "psc_version": (i32, []),
        "psc_last_error": (C.c_char_p, []),
        "psc_set_filter_route": (i32, [i32]),
        "psc_last_scan_route": (C.c_char_p, []),
        "psc_prepare": (i32, [vp, vp]),
        "psc_set_rotation": (i32, [vp, vp, i32]),
        "psc_rotate": (i32, [vp, vp, i64, vp, vp]),
        "psc_create": (i32, [C.POINTER(vp), i32, i32]),
        "psc_destroy": (None, [vp]),
        "psc_train_pq": (i32, [vp, vp, i64, i32, u64]),
        "psc_train_pq_device": (i32, [vp, vp, i64, i32, u64, i32, vp, vp]),
        "psc_optimize_index_assignment": (i32, [vp, i64, dbl, dbl, dbl, u64, vp, vp]),
        "psc_optimize_index_assignment_ranking": (i32, [vp, i64, dbl, dbl, u64, vp, vp]),
        "psc_set_codebook": (i32, [vp, vp]),
        "psc_get_codebook": (i32, [vp, vp]),
        "psc_encode": (i32, [vp, vp, i64, vp, vp]),
        "psc_build_lut": (i32, [vp, vp, i64, vp, vp, vp]),
        "psc_hamming_filter": (i32, [i32, vp, i64, vp, i64, i32, vp, vp, vp]),
        "psc_hamming_histogram": (i32, [i32, vp, i64, vp, i64, vp, vp]),
        "psc_threshold_for_rate": (i32, [vp, i32, dbl]),
        "psc_scan_workspace_bytes": (sz, [i32, i64, i64, i32]),
        "psc_scan": (i32, [i32, vp, vp, i64, vp, i64, i32, i32, vp, vp, vp, sz, vp]),
        "psc_scan_static": (i32, [i32, vp, vp, i64, vp, i64, i32, i32, vp, vp, vp]),
        "psc_search_workspace_bytes": (sz, [vp, i64, i64, i32]),
        "psc_search": (i32, [vp, vp, i64, vp, i64, i32, i32, vp, vp, vp, sz, vp]),
        "psc_knn_graph_workspace_bytes": (sz, [vp, i64, i32]),
        "psc_knn_graph": (i32, [vp, vp, vp, i64, i32, i32, vp, vp, vp, sz, vp]),
        "psc_ivf_train_coarse": (i32, [vp, vp, i64, i32, i32, u64]),
        "psc_ivf_train_coarse_device": (i32, [vp, vp, i64, i32, i32, u64, vp]),
        "psc_ivf_set_coarse": (i32, [vp, vp, i32]),
        "psc_ivf_get_coarse": (i32, [vp, vp]),
        "psc_ivf_assign_encode": (i32, [vp, vp, i64, vp, vp, vp]),
        "psc_ivf_set_lists": (i32, [vp, vp, vp, vp, i64]),
        "psc_ivf_search_workspace_bytes": (sz, [vp, i64, i32, i32]),
        "psc_ivf_search": (i32, [vp, vp, i64, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]),
        "psc_imi_set_coarse": (i32, [vp, vp, i32, vp, i32]),
        "psc_imi_assign_workspace_bytes": (sz, [vp, i64]),
        "psc_imi_assign_encode": (i32, [vp, vp, i64, vp, vp, vp, sz, vp]),
        "psc_imi_set_lists": (i32, [vp, vp, vp, vp, i64]),
        "psc_imi_search_workspace_bytes": (sz, [vp, i64, i32]),
        "psc_imi_search": (i32, [vp, vp, i64, i32, i64, i32, i32, vp, vp, vp, vp, vp, sz, vp]),
        "psc_workspace_status": (i32, [vp, vp]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def exported_symbols():
    """Names this binding expects the library to export."""
    _load()
    return ["psc_version", "psc_last_error", "psc_set_filter_route", "psc_last_scan_route", "psc_prepare", "psc_set_rotation", "psc_rotate", "psc_create", "psc_destroy", "psc_train_pq",
            "psc_train_pq_device", "psc_ivf_train_coarse_device",
            "psc_optimize_index_assignment", "psc_optimize_index_assignment_ranking", "psc_set_codebook", "psc_get_codebook", "psc_encode",
            "psc_build_lut", "psc_hamming_filter", "psc_hamming_histogram", "psc_threshold_for_rate",
            "psc_scan_workspace_bytes", "psc_scan", "psc_scan_static",
            "psc_search_workspace_bytes", "psc_search", "psc_knn_graph_workspace_bytes",
            "psc_knn_graph", "psc_ivf_train_coarse", "psc_ivf_set_coarse", "psc_ivf_get_coarse",
            "psc_ivf_assign_encode", "psc_ivf_set_lists", "psc_ivf_search_workspace_bytes",
            "psc_ivf_search", "psc_imi_set_coarse", "psc_imi_assign_workspace_bytes", "psc_imi_assign_encode",
            "psc_imi_set_lists", "psc_imi_search_workspace_bytes", "psc_imi_search", "psc_workspace_status"]


def _check(rc: int):
    if rc != 0:
        raise PscError(f"libpsc error {rc}: {_load().psc_last_error().decode()}")


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, dtype, name: str):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise PscError(f"{name}: expected a contiguous CUDA tensor of {dtype}")
    return C.c_void_p(t.data_ptr())


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def version() -> int:
    return _load().psc_version()


ROUTES = {"auto": 0, "popcount": 1, "mfma": 2}


def set_filter_route(route: str) -> None:
    """Force one of the two exact Hamming filters where both apply ("auto": the library's rule)."""
    _check(_load().psc_set_filter_route(ROUTES[route]))


def last_scan_route() -> str:
    """Kernel, tile shape, slices and workgroups of this thread's last scan."""
    return _load().psc_last_scan_route().decode()


class Index:
    """Owner of a product-quantizer codebook (host and device copies)."""

    def __init__(self, dim: int, m: int):
        lib = _load()
        self.dim, self.m, self.dsub = dim, m, dim // m if m else 0
        self.nlist = 0
        self._lists = None
        h = C.c_void_p()
        _check(lib.psc_create(C.byref(h), dim, m))
        self._h = h

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h is not None and _lib is not None:
            _lib.psc_destroy(h)

    # -- training, host side
    def train_pq(self, x: np.ndarray, iters: int = 20, seed: int = 0):
        x = np.ascontiguousarray(x, dtype=np.float32)
        assert x.ndim == 2 and x.shape[1] == self.dim
        _check(_load().psc_train_pq(self._h, x.ctypes.data_as(C.c_void_p), x.shape[0], iters, seed))

    def train_pq_device(self, x: torch.Tensor, iters: int = 20, seed: int = 0, from_current: bool = False):
        """Lloyd iterations on the GPU; returns the objective [iters, m] (float64)."""
        assert x.ndim == 2 and x.shape[1] == self.dim
        obj = np.empty((iters, self.m), dtype=np.float64)
        _check(_load().psc_train_pq_device(self._h, _dev(x, torch.float32, "x"), x.shape[0], iters, seed,
                                           PSC_START_CURRENT if from_current else PSC_START_SEEDED, obj.ctypes.data_as(C.c_void_p), _stream()))
        return obj

    def optimize_index_assignment(self, n_iter: int = 500_000, t0: float = 0.7,
                                  t_decay: float = 0.9 ** (1.0 / 500.0), alpha: float = 0.5,
                                  seed: int = 0):
        """Returns (pi [m,256] uint8, losses [m,2] float64 = before/after)."""
        pi = np.empty((self.m, 256), dtype=np.uint8)
        loss = np.empty((self.m, 2), dtype=np.float64)
        _check(_load().psc_optimize_index_assignment(self._h, n_iter, t0, t_decay, alpha, seed,
                                                     pi.ctypes.data_as(C.c_void_p),
                                                     loss.ctypes.data_as(C.c_void_p)))
        return pi, loss

    def optimize_index_assignment_ranking(self, n_iter: int = 500_000, t0: float = 0.7,
                                          t_decay: float = 0.9 ** (1.0 / 500.0), seed: int = 0):
        """The annealing on the ranking loss.  Returns (pi [m,256] uint8, losses [m,2] = before/after)."""
        pi = np.empty((self.m, 256), dtype=np.uint8)
        loss = np.empty((self.m, 2), dtype=np.float64)
        _check(_load().psc_optimize_index_assignment_ranking(self._h, n_iter, t0, t_decay, seed,
                                                             pi.ctypes.data_as(C.c_void_p),
                                                             loss.ctypes.data_as(C.c_void_p)))
        return pi, loss

    def set_codebook(self, cb: np.ndarray):
        cb = np.ascontiguousarray(cb, dtype=np.float32)
        assert cb.shape == (self.m, 256, self.dsub)
        _check(_load().psc_set_codebook(self._h, cb.ctypes.data_as(C.c_void_p)))

    def get_codebook(self) -> np.ndarray:
        cb = np.empty((self.m, 256, self.dsub), dtype=np.float32)
        _check(_load().psc_get_codebook(self._h, cb.ctypes.data_as(C.c_void_p)))
        return cb

    def set_rotation(self, r: np.ndarray):
        """Install the transformation r [dim, dim_in] applied by `rotate`."""
        r = np.ascontiguousarray(r, dtype=np.float32)
        assert r.ndim == 2 and r.shape[0] == self.dim
        _check(_load().psc_set_rotation(self._h, r.ctypes.data_as(C.c_void_p), r.shape[1]))
        self.dim_in = r.shape[1]

    def rotate(self, x: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
        """y [n, dim] = x [n, dim_in] . r^T."""
        n = x.shape[0]
        if out is None:
            out = torch.empty((n, self.dim), dtype=torch.float32, device=x.device)
        _check(_load().psc_rotate(self._h, _dev(x, torch.float32, "x"), n, _dev(out, torch.float32, "y"), _stream()))
        return out

    def prepare(self):
        """Upload the index's device image now, so that later calls neither allocate nor block."""
        _check(_load().psc_prepare(self._h, _stream()))

    # -- device operations
    def encode(self, x: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
        n = x.shape[0]
        if out is None:
            out = torch.empty((n, self.m), dtype=torch.uint8, device=x.device)
        _check(_load().psc_encode(self._h, _dev(x, torch.float32, "x"), n, _dev(out, torch.uint8, "codes"),
                                  _stream()))
        return out

    def build_lut(self, q: torch.Tensor, want_codes: bool = True):
        nq = q.shape[0]
        lut = torch.empty((nq, self.m, 256), dtype=torch.float32, device=q.device)
        qc = torch.empty((nq, self.m), dtype=torch.uint8, device=q.device) if want_codes else None
        _check(_load().psc_build_lut(self._h, _dev(q, torch.float32, "q"), nq, _dev(lut, torch.float32, "lut"),
                                     _dev(qc, torch.uint8, "qcodes") if want_codes else None, _stream()))
        return lut, qc

    def search(self, q: torch.Tensor, codes: torch.Tensor, ht: int, k: int, workspace=None, out=None):
        nq, n = q.shape[0], codes.shape[0]
        lib = _load()
        need = lib.psc_search_workspace_bytes(self._h, nq, n, k)
        if need == 0:
            _check(-1)
        ws = workspace if workspace is not None else _workspace(need, q.device)
        ids, dists = out if out is not None else (
            torch.empty((nq, k), dtype=torch.int64, device=q.device),
            torch.empty((nq, k), dtype=torch.float32, device=q.device))
        _check(lib.psc_search(self._h, _dev(q, torch.float32, "q"), nq, _dev(codes, torch.uint8, "codes"), n,
                              ht, k, _dev(ids, torch.int64, "ids"), _dev(dists, torch.float32, "dists"),
                              _dev(ws, torch.uint8, "workspace"), ws.numel(), _stream()))
        return ids, dists

    def knn_graph(self, x: torch.Tensor, codes: torch.Tensor, ht: int, k: int, workspace=None, out=None):
        """k nearest other rows for every row of x (ids [n,k] int64, dists [n,k] float32)."""
        n = x.shape[0]
        lib = _load()
        need = lib.psc_knn_graph_workspace_bytes(self._h, n, k)
        if need == 0:
            _check(-1)
        ws = workspace if workspace is not None else _workspace(need, x.device)
        ids, dists = out if out is not None else (
            torch.empty((n, k), dtype=torch.int64, device=x.device),
            torch.empty((n, k), dtype=torch.float32, device=x.device))
        _check(lib.psc_knn_graph(self._h, _dev(x, torch.float32, "x"), _dev(codes, torch.uint8, "codes"), n,
                                 ht, k, _dev(ids, torch.int64, "ids"), _dev(dists, torch.float32, "dists"),
                                 _dev(ws, torch.uint8, "workspace"), ws.numel(), _stream()))
        return ids, dists

    # -- inverted file
    def ivf_train_coarse(self, x: np.ndarray, nlist: int, iters: int = 10, seed: int = 0):
        x = np.ascontiguousarray(x, dtype=np.float32)
        assert x.ndim == 2 and x.shape[1] == self.dim
        _check(_load().psc_ivf_train_coarse(self._h, x.ctypes.data_as(C.c_void_p), x.shape[0], nlist, iters, seed))
        self.nlist = nlist

    def ivf_train_coarse_device(self, x: torch.Tensor, nlist: int, iters: int = 10, seed: int = 0):
        assert x.ndim == 2 and x.shape[1] == self.dim
        _check(_load().psc_ivf_train_coarse_device(self._h, _dev(x, torch.float32, "x"), x.shape[0], nlist, iters,
                                                   seed, _stream()))
        self.nlist = nlist

    def ivf_set_coarse(self, cent: np.ndarray):
        cent = np.ascontiguousarray(cent, dtype=np.float32)
        assert cent.ndim == 2 and cent.shape[1] == self.dim
        _check(_load().psc_ivf_set_coarse(self._h, cent.ctypes.data_as(C.c_void_p), cent.shape[0]))
        self.nlist = cent.shape[0]

    def ivf_get_coarse(self) -> np.ndarray:
        cent = np.empty((self.nlist, self.dim), dtype=np.float32)
        _check(_load().psc_ivf_get_coarse(self._h, cent.ctypes.data_as(C.c_void_p)))
        return cent

    def ivf_assign_encode(self, x: torch.Tensor, want_codes: bool = True):
        n = x.shape[0]
        list_no = torch.empty(n, dtype=torch.int32, device=x.device)
        codes = torch.empty((n, self.m), dtype=torch.uint8, device=x.device) if want_codes else None
        _check(_load().psc_ivf_assign_encode(self._h, _dev(x, torch.float32, "x"), n,
                                             _dev(list_no, torch.int32, "list_no"),
                                             _dev(codes, torch.uint8, "codes") if want_codes else None, _stream()))
        return list_no, codes

    def ivf_set_lists(self, offsets: torch.Tensor, codes: torch.Tensor, ids: torch.Tensor):
        """Borrow the caller's lists; the tensors are kept referenced by this object."""
        n = codes.shape[0]
        _check(_load().psc_ivf_set_lists(self._h, _dev(offsets, torch.int64, "offsets"),
                                         _dev(codes, torch.uint8, "codes"), _dev(ids, torch.int32, "ids"), n))
        self._lists = (offsets, codes, ids)

    def ivf_search_workspace_bytes(self, nq: int, nprobe: int, k: int) -> int:
        return int(_load().psc_ivf_search_workspace_bytes(self._h, nq, nprobe, k))

    def ivf_search(self, q: torch.Tensor, nprobe: int, ht: int, k: int, workspace=None, out=None,
                   want_debug: bool = False):
        nq = q.shape[0]
        lib = _load()
        need = lib.psc_ivf_search_workspace_bytes(self._h, nq, nprobe, k)
        if need == 0:
            _check(-1)
        ws = workspace if workspace is not None else _workspace(need, q.device)
        ids, dists = out if out is not None else (
            torch.empty((nq, k), dtype=torch.int64, device=q.device),
            torch.empty((nq, k), dtype=torch.float32, device=q.device))
        npb = min(nprobe, self.nlist)
        probed = torch.empty((nq, npb), dtype=torch.int32, device=q.device) if want_debug else None
        qcodes = torch.empty((nq, npb, self.m), dtype=torch.uint8, device=q.device) if want_debug else None
        _check(lib.psc_ivf_search(self._h, _dev(q, torch.float32, "q"), nq, nprobe, ht, k,
                                  _dev(ids, torch.int64, "ids"), _dev(dists, torch.float32, "dists"),
                                  _dev(probed, torch.int32, "probed") if want_debug else None,
                                  _dev(qcodes, torch.uint8, "qcodes") if want_debug else None,
                                  _dev(ws, torch.uint8, "workspace"), ws.numel(), _stream()))
        return (ids, dists, probed, qcodes) if want_debug else (ids, dists)

    # -- inverted multi-index
    def imi_set_coarse(self, c1: np.ndarray, c2: np.ndarray):
        c1, c2 = np.ascontiguousarray(c1, dtype=np.float32), np.ascontiguousarray(c2, dtype=np.float32)
        assert c1.ndim == 2 and c2.ndim == 2 and c1.shape[1] == self.dim // 2 and c2.shape[1] == self.dim // 2
        _check(_load().psc_imi_set_coarse(self._h, c1.ctypes.data_as(C.c_void_p), c1.shape[0],
                                          c2.ctypes.data_as(C.c_void_p), c2.shape[0]))
        self.imi_k = (c1.shape[0], c2.shape[0])
        self._imi_c1, self._imi_c2 = c1, c2

    def imi_assign_workspace_bytes(self, n: int) -> int:
        return int(_load().psc_imi_assign_workspace_bytes(self._h, n))

    def imi_assign_encode(self, x: torch.Tensor, want_codes: bool = True, workspace=None):
        n = x.shape[0]
        lib = _load()
        ws = workspace if workspace is not None else _workspace(lib.psc_imi_assign_workspace_bytes(self._h, n), x.device)
        cell = torch.empty(n, dtype=torch.int32, device=x.device)
        codes = torch.empty((n, self.m), dtype=torch.uint8, device=x.device) if want_codes else None
        _check(lib.psc_imi_assign_encode(self._h, _dev(x, torch.float32, "x"), n, _dev(cell, torch.int32, "cell"),
                                         _dev(codes, torch.uint8, "codes") if want_codes else None,
                                         _dev(ws, torch.uint8, "workspace"), ws.numel(), _stream()))
        return cell, codes

    def imi_set_lists(self, offsets: torch.Tensor, codes: torch.Tensor, ids: torch.Tensor):
        """Borrow the caller's cell lists; the tensors are kept referenced by this object."""
        _check(_load().psc_imi_set_lists(self._h, _dev(offsets, torch.int64, "offsets"), _dev(codes, torch.uint8, "codes"),
                                         _dev(ids, torch.int32, "ids"), codes.shape[0]))
        self._imi_lists = (offsets, codes, ids)

    def imi_search_workspace_bytes(self, nq: int, max_lists: int) -> int:
        return int(_load().psc_imi_search_workspace_bytes(self._h, nq, max_lists))

    def imi_search(self, q: torch.Tensor, max_lists: int, max_codes: int, ht: int, k: int, workspace=None, out=None,
                   want_debug: bool = False):
        nq = q.shape[0]
        lib = _load()
        need = lib.psc_imi_search_workspace_bytes(self._h, nq, max_lists)
        if need == 0:
            _check(-1)
        ws = workspace if workspace is not None else _workspace(need, q.device)
        ids, dists = out if out is not None else (
            torch.empty((nq, k), dtype=torch.int64, device=q.device),
            torch.empty((nq, k), dtype=torch.float32, device=q.device))
        cells = torch.empty((nq, max_lists), dtype=torch.int32, device=q.device) if want_debug else None
        qcodes = torch.empty((nq, max_lists, self.m), dtype=torch.uint8, device=q.device) if want_debug else None
        _check(lib.psc_imi_search(self._h, _dev(q, torch.float32, "q"), nq, max_lists, max_codes, ht, k,
                                  _dev(ids, torch.int64, "ids"), _dev(dists, torch.float32, "dists"),
                                  _dev(cells, torch.int32, "cells") if want_debug else None,
                                  _dev(qcodes, torch.uint8, "qcodes") if want_debug else None,
                                  _dev(ws, torch.uint8, "workspace"), ws.numel(), _stream()))
        return (ids, dists, cells, qcodes) if want_debug else (ids, dists)

    def knn_graph_workspace_bytes(self, n: int, k: int) -> int:
        return int(_load().psc_knn_graph_workspace_bytes(self._h, n, k))

    def search_workspace_bytes(self, nq: int, n: int, k: int) -> int:
        return int(_load().psc_search_workspace_bytes(self._h, nq, n, k))


def scan_workspace_bytes(m: int, nq: int, n: int, k: int) -> int:
    return int(_load().psc_scan_workspace_bytes(m, nq, n, k))


def scan(lut: torch.Tensor, qcodes: torch.Tensor, codes: torch.Tensor, ht: int, k: int,
         workspace=None, out=None):
    """Fused Hamming filter + ADC + top-k.  Returns (ids [nq,k] int64, dists [nq,k] float32)."""
    lib = _load()
    nq, m = qcodes.shape
    n = codes.shape[0]
    need = lib.psc_scan_workspace_bytes(m, nq, n, k)
    if need == 0:
        _check(lib.psc_scan(m, None, None, nq, None, n, ht, k, None, None, None, 0, None) or -1)
    ws = workspace if workspace is not None else _workspace(need, qcodes.device)
    ids, dists = out if out is not None else (
        torch.empty((nq, k), dtype=torch.int64, device=qcodes.device),
        torch.empty((nq, k), dtype=torch.float32, device=qcodes.device))
    _check(lib.psc_scan(m, _dev(lut, torch.float32, "lut"), _dev(qcodes, torch.uint8, "qcodes"), nq,
                        _dev(codes, torch.uint8, "codes"), n, ht, k, _dev(ids, torch.int64, "ids"),
                        _dev(dists, torch.float32, "dists"), _dev(ws, torch.uint8, "workspace"),
                        ws.numel(), _stream()))
    return ids, dists


PSC_STATIC_SCRATCH_BYTES = 32 << 20


def scan_static(lut: torch.Tensor, qcodes: torch.Tensor, codes: torch.Tensor, ht: int, k: int, out):
    """`scan` on the library's static scratch array: no workspace, no allocation (results go to
    the caller's `out` = (ids [nq,k] int64, dists [nq,k] float32))."""
    nq, m = qcodes.shape
    ids, dists = out
    _check(_load().psc_scan_static(m, _dev(lut, torch.float32, "lut"), _dev(qcodes, torch.uint8, "qcodes"), nq,
                                   _dev(codes, torch.uint8, "codes"), codes.shape[0], ht, k,
                                   _dev(ids, torch.int64, "ids"), _dev(dists, torch.float32, "dists"), _stream()))
    return ids, dists


def hamming_filter(qcodes: torch.Tensor, codes: torch.Tensor, ht: int, want_distances: bool = False):
    """Per-query survivor counts (int64 [nq]) and optionally all distances (uint8 [nq,n])."""
    nq, m = qcodes.shape
    n = codes.shape[0]
    nsurv = torch.empty(nq, dtype=torch.int64, device=qcodes.device)
    hd = torch.empty((nq, n), dtype=torch.uint8, device=qcodes.device) if want_distances else None
    _check(_load().psc_hamming_filter(m, _dev(qcodes, torch.uint8, "qcodes"), nq,
                                      _dev(codes, torch.uint8, "codes"), n, ht,
                                      _dev(nsurv, torch.int64, "nsurv"),
                                      _dev(hd, torch.uint8, "hdist") if want_distances else None, _stream()))
    return (nsurv, hd) if want_distances else nsurv


def hamming_histogram(qcodes: torch.Tensor, codes: torch.Tensor) -> torch.Tensor:
    """Number of (query code, code) pairs at every Hamming distance 0..8m (int64 [8m+1])."""
    nq, m = qcodes.shape
    hist = torch.empty(8 * m + 1, dtype=torch.int64, device=qcodes.device)
    _check(_load().psc_hamming_histogram(m, _dev(qcodes, torch.uint8, "qcodes"), nq,
                                         _dev(codes, torch.uint8, "codes"), codes.shape[0],
                                         _dev(hist, torch.int64, "hist"), _stream()))
    return hist


def threshold_for_rate(hist, max_keep_fraction: float) -> int:
    """Largest ht that keeps at most `max_keep_fraction` of the pairs of a histogram (-1: none)."""
    h = np.ascontiguousarray(hist.cpu().numpy() if isinstance(hist, torch.Tensor) else hist, dtype=np.int64)
    if h.size < 2 or h.sum() <= 0:
        raise PscError("empty histogram")
    return int(_load().psc_threshold_for_rate(h.ctypes.data_as(C.c_void_p), h.size - 1, float(max_keep_fraction)))


def workspace_status(ws: torch.Tensor) -> None:
    _check(_load().psc_workspace_status(_dev(ws, torch.uint8, "workspace"), _stream()))
