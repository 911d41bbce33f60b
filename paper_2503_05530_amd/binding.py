"""ctypes binding of libproximity.so (the C ABI in include/proximity.h).

Argument marshalling only: every step of the retrieval path runs in the HIP
library.  PyTorch supplies device memory and the stream.  There is no CPU
fallback: if the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np
import torch

from .build import LIB_PATH

OK = 0
ERR_INVALID_ARG, ERR_K_MISMATCH, ERR_BATCH_TOO_LARGE, ERR_BAD_TAU, ERR_HIP, ERR_OOM = -1, -2, -3, -4, -5, -6
DTYPE_F32, DTYPE_BF16 = 0, 1
POLICY_FIFO, POLICY_LRU = 0, 1
METRIC_L2, METRIC_IP, METRIC_COSINE = 0, 1, 2
ABI_VERSION = 9
FLAG_NO_ROUNDED_SCAN = 1
MAX_K, MAX_DIM, MAX_BATCH, MAX_CAPACITY = 240, 4096, 8192, 1 << 20   # PROXIMITY_MAX_* of the header
STATIC_MAX_DOCS, STATIC_MAX_QUERIES = 1 << 18, 4                      # PROXIMITY_STATIC_MAX_* of the header


class ProximityConfig(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("dim", C.c_uint32), ("corpus", C.c_void_p),
                ("n_docs", C.c_uint64), ("corpus_dtype", C.c_uint32), ("capacity", C.c_uint32),
                ("k", C.c_uint32), ("policy", C.c_uint32), ("max_batch", C.c_uint32), ("device", C.c_int32),
                ("rerank_factor", C.c_uint32), ("lsh_bits", C.c_uint32), ("lsh_planes", C.c_void_p),
                ("metric", C.c_uint32), ("flags", C.c_uint32)]


class ProximityStats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("queries", "hits", "misses", "inserts", "evictions", "size",
                                          "inbatch_hits", "dense_resolves", "slack_exhausted",
                                          "slack_unresolved", "probe_workspace_bytes", "coarse_scan_calls",
                                          "coarse_scan_fails")] + [("reserved", C.c_uint64 * 3)]


class ProximityLaunch(C.Structure):
    _fields_ = [("call", C.c_uint32), ("first_query", C.c_uint32), ("n_queries", C.c_uint32), ("ms", C.c_float),
                ("kind", C.c_uint32)]


LAUNCH_SCAN, LAUNCH_PROBE = 0, 1


if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build the HIP library first "
        "(python -c 'import __graft_entry__ as g; g.build()'). There is no CPU fallback.")

lib = C.CDLL(LIB_PATH)

_H = C.c_void_p
lib.proximity_abi_version.restype = C.c_uint32
lib.proximity_abi_version.argtypes = []
lib.proximity_score_error_bound.restype = C.c_double
lib.proximity_score_error_bound.argtypes = [C.c_uint32, C.c_uint32, C.c_double, C.c_double]
lib.proximity_coarse_score_error.restype = C.c_double
lib.proximity_coarse_score_error.argtypes = [C.c_uint32, C.c_uint32, C.c_double, C.c_double]
lib.proximity_rounded_scan_list_length.restype = C.c_uint32
lib.proximity_rounded_scan_list_length.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint64]
lib.proximity_probe_row_ranges.restype = C.c_uint32
lib.proximity_probe_row_ranges.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
                                           C.POINTER(C.c_uint32), C.c_uint32]
lib.proximity_last_error.restype = C.c_char_p
lib.proximity_last_error.argtypes = [_H]
lib.proximity_create.restype = C.c_int
lib.proximity_create.argtypes = [C.POINTER(ProximityConfig), C.POINTER(_H)]
lib.proximity_destroy.restype = None
lib.proximity_destroy.argtypes = [_H]
lib.proximity_search_batch.restype = C.c_int
lib.proximity_search_batch.argtypes = [_H, C.c_void_p, C.c_uint32, C.c_uint32, C.c_float, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p]
lib.proximity_knn_batch.restype = C.c_int
lib.proximity_knn_batch.argtypes = [_H, C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p]
lib.proximity_knn_static.restype = C.c_int
lib.proximity_knn_static.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p, C.c_uint32,
                                     C.c_uint32, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
lib.proximity_stats.restype = C.c_int
lib.proximity_stats.argtypes = [_H, C.POINTER(ProximityStats)]
lib.proximity_cache_dump.restype = C.c_int
lib.proximity_cache_dump.argtypes = [_H, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_uint32)]
lib.proximity_clear.restype = C.c_int
lib.proximity_clear.argtypes = [_H]
lib.proximity_profile_start.restype = C.c_int
lib.proximity_profile_start.argtypes = [_H]
lib.proximity_profile_stop.restype = C.c_int
lib.proximity_profile_stop.argtypes = [_H, C.POINTER(ProximityLaunch), C.c_uint32, C.POINTER(C.c_uint32)]

EXPORTED = ("proximity_abi_version", "proximity_score_error_bound", "proximity_coarse_score_error", "proximity_rounded_scan_list_length", "proximity_probe_row_ranges", "proximity_last_error", "proximity_create", "proximity_destroy",
            "proximity_search_batch", "proximity_knn_batch", "proximity_knn_static", "proximity_stats", "proximity_cache_dump",
            "proximity_clear", "proximity_profile_start", "proximity_profile_stop")


class ProximityError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"proximity error {code}: {message}")
        self.code = code


def last_error(handle=None) -> str:
    msg = lib.proximity_last_error(handle)
    return msg.decode() if msg else ""


def proximity_abi_version() -> int:
    return int(lib.proximity_abi_version())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def proximity_knn_static(corpus: torch.Tensor, queries: torch.Tensor, k: int, out_ids: torch.Tensor,
                         out_dists: Optional[torch.Tensor] = None, metric: int = METRIC_L2,
                         stream: Optional[torch.cuda.Stream] = None) -> None:
    """The index search without an instance and without any allocation (proximity_knn_static): the caller
    passes every buffer, outputs included."""
    dtype = DTYPE_BF16 if corpus.dtype == torch.bfloat16 else DTYPE_F32
    dev = corpus.device
    s = torch.cuda.current_stream(dev) if stream is None else stream
    rc = lib.proximity_knn_static(_ptr(corpus), corpus.shape[0], corpus.shape[1], dtype, int(metric), _ptr(queries),
                                  queries.shape[0], int(k), _ptr(out_ids), _ptr(out_dists),
                                  dev.index if dev.index is not None else 0, C.c_void_p(s.cuda_stream))
    if rc != OK:
        raise ProximityError(rc, last_error(None))


class Proximity:
    """One cache-plus-index instance.  Method names follow the C entry points."""

    def __init__(self, corpus: Optional[torch.Tensor], dim: int, capacity: int, k: int, policy: int,
                 max_batch: int, device: Optional[torch.device] = None, rerank_factor: int = 1,
                 lsh_planes: Optional[torch.Tensor] = None, metric: int = METRIC_L2, flags: int = 0):
        """``lsh_planes`` (device float32 [L][dim]) selects the bucketed cache of Section 3.2: 2^L buckets of
        ``capacity`` entries each.  ``metric`` is the index's distance function (METRIC_*), ``flags`` a sum of
        FLAG_*."""
        if corpus is not None:
            if not corpus.is_cuda or not corpus.is_contiguous() or corpus.dim() != 2:
                raise ValueError("corpus must be a contiguous 2-D device tensor")
            if corpus.dtype == torch.float32:
                dtype = DTYPE_F32
            elif corpus.dtype == torch.bfloat16:
                dtype = DTYPE_BF16
            else:
                raise ValueError("corpus must be float32 or bfloat16")
            if corpus.shape[1] != dim:
                raise ValueError("corpus width differs from dim")
            device = corpus.device
            n_docs = corpus.shape[0]
        else:
            dtype, n_docs = DTYPE_F32, 0
            device = torch.device("cuda:0") if device is None else torch.device(device)
        self.device = device
        self.corpus = corpus          # keeps the borrowed memory alive
        self.dim, self.capacity, self.k, self.policy, self.max_batch = dim, capacity, k, policy, max_batch
        self.rerank_factor = max(1, int(rerank_factor))
        self.lsh_bits = 0
        if lsh_planes is not None and lsh_planes.shape[0] > 0:
            if (not lsh_planes.is_cuda) or lsh_planes.dtype != torch.float32 or not lsh_planes.is_contiguous() \
                    or lsh_planes.dim() != 2 or lsh_planes.shape[1] != dim:
                raise ValueError("lsh_planes must be a contiguous float32 device tensor [L][dim]")
            self.lsh_bits = int(lsh_planes.shape[0])
        self.slots = capacity << self.lsh_bits if capacity > 0 else 0
        cfg = ProximityConfig(C.sizeof(ProximityConfig), dim, corpus.data_ptr() if corpus is not None else None,
                              n_docs, dtype, capacity, k, policy, max_batch,
                              device.index if device.index is not None else 0, int(rerank_factor), self.lsh_bits,
                              lsh_planes.data_ptr() if self.lsh_bits else None, int(metric), int(flags))
        self.metric = int(metric)
        self.handle = _H()
        rc = lib.proximity_create(C.byref(cfg), C.byref(self.handle))
        if rc != OK:
            raise ProximityError(rc, last_error(None))

    # -- the calls of the C ABI ------------------------------------------------
    def search_batch(self, queries: torch.Tensor, tau: float, out_ids=None, out_dists=None, out_hit=None,
                     want_dists: bool = True, stream: Optional[torch.cuda.Stream] = None):
        n = queries.shape[0]
        self._check_queries(queries)
        if out_ids is None:
            out_ids = torch.empty((n, self.k), dtype=torch.int64, device=self.device)
        if out_dists is None and want_dists:
            out_dists = torch.empty((n, self.k), dtype=torch.float32, device=self.device)
        if out_hit is None:
            out_hit = torch.empty((n,), dtype=torch.uint8, device=self.device)
        s = torch.cuda.current_stream(self.device) if stream is None else stream
        rc = lib.proximity_search_batch(self.handle, _ptr(queries), n, self.k, float(tau), _ptr(out_ids),
                                        _ptr(out_dists), _ptr(out_hit), C.c_void_p(s.cuda_stream))
        self._check(rc)
        return out_ids, out_dists, out_hit

    def knn_batch(self, queries: torch.Tensor, out_ids=None, out_dists=None,
                  stream: Optional[torch.cuda.Stream] = None):
        n = queries.shape[0]
        self._check_queries(queries)
        if out_ids is None:
            out_ids = torch.empty((n, self.k), dtype=torch.int64, device=self.device)
        if out_dists is None:
            out_dists = torch.empty((n, self.k), dtype=torch.float32, device=self.device)
        s = torch.cuda.current_stream(self.device) if stream is None else stream
        rc = lib.proximity_knn_batch(self.handle, _ptr(queries), n, self.k, _ptr(out_ids), _ptr(out_dists),
                                     C.c_void_p(s.cuda_stream))
        self._check(rc)
        return out_ids, out_dists

    def stats(self) -> dict:
        st = ProximityStats()
        self._check(lib.proximity_stats(self.handle, C.byref(st)))
        return {n: int(getattr(st, n)) for n, _ in ProximityStats._fields_ if n != "reserved"}

    def cache_dump(self, want_keys: bool = False, want_ids: bool = False):
        rows = max(self.slots, 1)
        seq = np.zeros(rows, dtype=np.uint64)
        keys = np.zeros((rows, self.dim), dtype=np.float32) if want_keys else None
        ids = np.zeros((rows, self.k * self.rerank_factor), dtype=np.int64) if want_ids else None
        n_live = C.c_uint32(0)
        rc = lib.proximity_cache_dump(self.handle, seq.ctypes.data_as(C.c_void_p),
                                      keys.ctypes.data_as(C.c_void_p) if want_keys else None,
                                      ids.ctypes.data_as(C.c_void_p) if want_ids else None, C.byref(n_live))
        self._check(rc)
        m = n_live.value
        return (seq[:m].astype(np.int64), keys[:m] if want_keys else None, ids[:m] if want_ids else None)

    def clear(self):
        self._check(lib.proximity_clear(self.handle))

    def profile_start(self):
        self._check(lib.proximity_profile_start(self.handle))

    def profile_stop(self, cap: int = 8192, kind: int = LAUNCH_SCAN):
        rec = (ProximityLaunch * cap)()
        n = C.c_uint32(0)
        self._check(lib.proximity_profile_stop(self.handle, rec, cap, C.byref(n)))
        return [(r.call, r.first_query, r.n_queries, r.ms) for r in rec[: n.value] if r.kind == kind]

    def close(self):
        if getattr(self, "handle", None):
            lib.proximity_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- helpers ---------------------------------------------------------------
    def _check_queries(self, q: torch.Tensor):
        if (not q.is_cuda) or q.dtype != torch.float32 or not q.is_contiguous() or q.dim() != 2 \
                or q.shape[1] != self.dim:
            raise ValueError("queries must be a contiguous float32 device tensor [n][dim]")

    def _check(self, rc: int):
        if rc != OK:
            raise ProximityError(rc, last_error(self.handle))
