"""ctypes binding for ``libiccache.so``: same entry points as ``include/iccache.h``.

Argument marshalling only.  Tensors supply device pointers; the current torch
stream supplies the ``hipStream_t``.  Every step of the search runs in the
library's kernels.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libiccache.so")

STORE_BF16 = 0
STORE_FP8_E4M3 = 1
IC_MAX_K = 128
IC_ARENA_ALIGN = 256

EXPORTS = (
    "ic_workspace_bytes", "ic_index_create", "ic_index_append", "ic_search", "ic_search_static", "ic_index_destroy",
    "ic_index_size", "ic_index_set_stream", "ic_index_store_view", "ic_index_set_timing", "ic_index_set_tuning",
    "ic_index_scan_time_ms", "ic_index_tiled_scan_counts", "ic_status_string",
    "ic_index_set_utility", "ic_index_scale_utility", "ic_index_invalidate", "ic_index_compact",
    "ic_search_threshold", "ic_self_search", "ic_index_set_domains", "ic_search_domains",
    "ic_ivf_workspace_bytes", "ic_ivf_create", "ic_ivf_destroy", "ic_ivf_set_centroids", "ic_ivf_assign",
    "ic_ivf_set_assignment", "ic_ivf_update_centroids", "ic_ivf_train", "ic_ivf_search", "ic_ivf_view",
)

_lib = None


class ICError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load_library().ic_status_string(status).decode()
        super().__init__(f"{where}: {msg} (ic_status {status})")


def lib_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load ``libiccache.so`` (built by ``paper_2501_12689_amd.build``); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2501_12689_amd.build`; "
            "there is no fallback path")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    L.ic_workspace_bytes.restype = ctypes.c_size_t
    L.ic_workspace_bytes.argtypes = [i32, ctypes.c_int, i64, i64, i32]
    L.ic_index_create.restype = ctypes.c_int
    L.ic_index_create.argtypes = [ctypes.POINTER(vp), i32, ctypes.c_int, i64, i64, i32, vp,
                                  ctypes.c_size_t, vp]
    L.ic_index_append.restype = ctypes.c_int
    L.ic_index_append.argtypes = [vp, vp, vp, i64, ctypes.POINTER(i64)]
    L.ic_search.restype = ctypes.c_int
    L.ic_search.argtypes = [vp, vp, i64, i32, f32, vp, vp, vp]
    L.ic_search_static.restype = ctypes.c_int
    L.ic_search_static.argtypes = [vp, vp, i64, i32, f32, vp, vp, vp]
    L.ic_search_threshold.restype = ctypes.c_int
    L.ic_search_threshold.argtypes = [vp, vp, i64, i32, f32, vp, f32, vp, vp, vp]
    L.ic_self_search.restype = ctypes.c_int
    L.ic_self_search.argtypes = [vp, i64, i64, i32, f32, vp, vp, vp]
    L.ic_index_destroy.restype = ctypes.c_int
    L.ic_index_destroy.argtypes = [vp]
    L.ic_index_size.restype = i64
    L.ic_index_size.argtypes = [vp]
    L.ic_index_set_stream.restype = ctypes.c_int
    L.ic_index_set_stream.argtypes = [vp, vp]
    L.ic_index_store_view.restype = ctypes.c_int
    L.ic_index_store_view.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(i64),
                                      ctypes.POINTER(vp), ctypes.POINTER(vp)]
    L.ic_index_set_timing.restype = ctypes.c_int
    L.ic_index_set_timing.argtypes = [vp, ctypes.c_int]
    L.ic_index_set_tuning.restype = ctypes.c_int
    L.ic_index_set_tuning.argtypes = [vp, i32, i32]
    L.ic_index_scan_time_ms.restype = ctypes.c_int
    L.ic_index_scan_time_ms.argtypes = [vp, ctypes.POINTER(f32), ctypes.POINTER(i64)]
    L.ic_index_tiled_scan_counts.restype = ctypes.c_int
    L.ic_index_tiled_scan_counts.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    L.ic_index_set_domains.restype = ctypes.c_int
    L.ic_index_set_domains.argtypes = [vp, vp, vp, i64]
    L.ic_search_domains.restype = ctypes.c_int
    L.ic_search_domains.argtypes = [vp, vp, i64, i32, f32, vp, vp, vp, vp]
    L.ic_index_set_utility.restype = ctypes.c_int
    L.ic_index_set_utility.argtypes = [vp, vp, vp, i64]
    L.ic_index_scale_utility.restype = ctypes.c_int
    L.ic_index_scale_utility.argtypes = [vp, f32]
    L.ic_index_invalidate.restype = ctypes.c_int
    L.ic_index_invalidate.argtypes = [vp, vp, i64]
    L.ic_index_compact.restype = ctypes.c_int
    L.ic_index_compact.argtypes = [vp, vp, ctypes.POINTER(i64)]
    L.ic_ivf_workspace_bytes.restype = ctypes.c_size_t
    L.ic_ivf_workspace_bytes.argtypes = [vp, i32, i32]
    L.ic_ivf_create.restype = ctypes.c_int
    L.ic_ivf_create.argtypes = [ctypes.POINTER(vp), vp, i32, i32, vp, ctypes.c_size_t]
    for name, args in (("ic_ivf_destroy", [vp]), ("ic_ivf_set_centroids", [vp, vp]), ("ic_ivf_assign", [vp]),
                       ("ic_ivf_set_assignment", [vp, vp]), ("ic_ivf_update_centroids", [vp]),
                       ("ic_ivf_train", [vp, i32]),
                       ("ic_ivf_search", [vp, vp, i64, i32, i32, f32, vp, vp]),
                       ("ic_ivf_view", [vp] + [ctypes.POINTER(vp)] * 5)):
        getattr(L, name).restype = ctypes.c_int
        getattr(L, name).argtypes = args
    L.ic_status_string.restype = ctypes.c_char_p
    L.ic_status_string.argtypes = [ctypes.c_int]
    _lib = L
    return L


def _check(status: int, where: str) -> None:
    if status != 0:
        raise ICError(status, where)


def _dev_ptr(t: Optional[torch.Tensor], dtype, name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous {dtype} tensor on the GPU")
    return t.data_ptr()


# ---- the four calls of the ABI, on raw handles --------------------------------

def ic_workspace_bytes(d: int, store: int, capacity_rows: int, max_queries: int, max_k: int) -> int:
    return int(load_library().ic_workspace_bytes(d, store, capacity_rows, max_queries, max_k))


def ic_index_create(d: int, store: int, capacity_rows: int, max_queries: int, max_k: int,
                    arena: torch.Tensor, stream: Optional[int] = None) -> int:
    """Returns the opaque handle.  ``arena`` is a uint8 GPU tensor the caller keeps alive."""
    L = load_library()
    ptr = _dev_ptr(arena, torch.uint8, "arena")
    if stream is None:
        stream = torch.cuda.current_stream(arena.device).cuda_stream
    h = ctypes.c_void_p()
    _check(L.ic_index_create(ctypes.byref(h), d, store, capacity_rows, max_queries, max_k, ptr,
                             arena.numel(), stream), "ic_index_create")
    return h.value


def ic_index_append(handle: int, emb: torch.Tensor, util: Optional[torch.Tensor] = None) -> int:
    """Append ``emb`` [n,d] fp32 (and ``util`` [n] fp32); returns the first new id."""
    L = load_library()
    first = ctypes.c_int64(-1)
    n = emb.shape[0] if emb is not None else 0
    _check(L.ic_index_append(handle, _dev_ptr(emb, torch.float32, "emb"),
                             _dev_ptr(util, torch.float32, "util"), n, ctypes.byref(first)),
           "ic_index_append")
    return first.value


def ic_search(handle: int, queries: torch.Tensor, k: int, lam: float = 0.0,
              mask: Optional[torch.Tensor] = None, out_scores: Optional[torch.Tensor] = None,
              out_ids: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Top-k of ``cos + lam*utility`` over valid rows: (scores fp32 [Q,k], ids int64 [Q,k])."""
    L = load_library()
    Q = queries.shape[0]
    if out_scores is None:
        out_scores = torch.empty((Q, k), dtype=torch.float32, device=queries.device)
    if out_ids is None:
        out_ids = torch.empty((Q, k), dtype=torch.int64, device=queries.device)
    _check(L.ic_search(handle, _dev_ptr(queries, torch.float32, "queries"), Q, k, float(lam),
                       _dev_ptr(mask, torch.uint8, "mask"),
                       _dev_ptr(out_scores, torch.float32, "out_scores"),
                       _dev_ptr(out_ids, torch.int64, "out_ids")), "ic_search")
    return out_scores, out_ids


def ic_search_static(handle: int, queries: torch.Tensor, k: int, lam: float, mask: Optional[torch.Tensor],
                     out_scores: torch.Tensor, out_ids: torch.Tensor) -> None:
    """``ic_search`` with the library's static scratch; the caller passes the outputs (nothing is allocated)."""
    _check(load_library().ic_search_static(handle, _dev_ptr(queries, torch.float32, "queries"), queries.shape[0], k,
                                           float(lam), _dev_ptr(mask, torch.uint8, "mask"),
                                           _dev_ptr(out_scores, torch.float32, "out_scores"),
                                           _dev_ptr(out_ids, torch.int64, "out_ids")), "ic_search_static")


def ic_search_threshold(handle: int, queries: torch.Tensor, k: int, min_score: float, lam: float = 0.0,
                        mask: Optional[torch.Tensor] = None):
    """ic_search that keeps only entries with score >= min_score: (scores, ids, counts int32 [Q])."""
    L = load_library()
    Q = queries.shape[0]
    out_scores = torch.empty((Q, k), dtype=torch.float32, device=queries.device)
    out_ids = torch.empty((Q, k), dtype=torch.int64, device=queries.device)
    counts = torch.empty((Q,), dtype=torch.int32, device=queries.device)
    _check(L.ic_search_threshold(handle, _dev_ptr(queries, torch.float32, "queries"), Q, k, float(lam),
                                 _dev_ptr(mask, torch.uint8, "mask"), float(min_score),
                                 _dev_ptr(out_scores, torch.float32, "out_scores"),
                                 _dev_ptr(out_ids, torch.int64, "out_ids"),
                                 _dev_ptr(counts, torch.int32, "counts")), "ic_search_threshold")
    return out_scores, out_ids, counts


def ic_search_domains(handle: int, queries: torch.Tensor, k: int, query_domain: torch.Tensor, lam: float = 0.0,
                      mask: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """ic_search in which query j sees only the rows of domain 0 or ``query_domain[j]`` (int32 [Q])."""
    L = load_library()
    Q = queries.shape[0]
    if query_domain.numel() != Q:
        raise ValueError("ic_search_domains: one domain per query expected")
    out_scores = torch.empty((Q, k), dtype=torch.float32, device=queries.device)
    out_ids = torch.empty((Q, k), dtype=torch.int64, device=queries.device)
    _check(L.ic_search_domains(handle, _dev_ptr(queries, torch.float32, "queries"), Q, k, float(lam),
                               _dev_ptr(mask, torch.uint8, "mask"),
                               _dev_ptr(query_domain, torch.int32, "query_domain"),
                               _dev_ptr(out_scores, torch.float32, "out_scores"),
                               _dev_ptr(out_ids, torch.int64, "out_ids")), "ic_search_domains")
    return out_scores, out_ids


def ic_self_search(handle: int, first_row: int, count: int, k: int, lam: float, mask: Optional[torch.Tensor],
                   device) -> Tuple[torch.Tensor, torch.Tensor]:
    """Top-k of the stored rows [first_row, first_row + count) among all other rows."""
    out_scores = torch.empty((count, k), dtype=torch.float32, device=device)
    out_ids = torch.empty((count, k), dtype=torch.int64, device=device)
    _check(load_library().ic_self_search(handle, first_row, count, k, float(lam),
                                         _dev_ptr(mask, torch.uint8, "mask"),
                                         _dev_ptr(out_scores, torch.float32, "out_scores"),
                                         _dev_ptr(out_ids, torch.int64, "out_ids")), "ic_self_search")
    return out_scores, out_ids


def ic_index_destroy(handle: int) -> None:
    _check(load_library().ic_index_destroy(handle), "ic_index_destroy")


def ic_index_set_utility(handle: int, ids: torch.Tensor, util: torch.Tensor) -> None:
    """utility[ids[j]] = util[j] (ids int64 [n], util fp32 [n], both on the GPU)."""
    _check(load_library().ic_index_set_utility(handle, _dev_ptr(ids, torch.int64, "ids"),
                                               _dev_ptr(util, torch.float32, "util"), ids.numel()),
           "ic_index_set_utility")


def ic_index_set_domains(handle: int, ids: torch.Tensor, domains: torch.Tensor) -> None:
    """domain[ids[j]] = domains[j] (ids int64 [n], domains int32 [n], both on the GPU)."""
    if ids.numel() != domains.numel():
        raise ValueError("ic_index_set_domains: one domain per id expected")
    _check(load_library().ic_index_set_domains(handle, _dev_ptr(ids, torch.int64, "ids"),
                                               _dev_ptr(domains, torch.int32, "domains"), ids.numel()),
           "ic_index_set_domains")


def ic_index_scale_utility(handle: int, factor: float) -> None:
    _check(load_library().ic_index_scale_utility(handle, float(factor)), "ic_index_scale_utility")


def ic_index_invalidate(handle: int, ids: torch.Tensor) -> None:
    """Mark rows as evicted; later searches never return them."""
    _check(load_library().ic_index_invalidate(handle, _dev_ptr(ids, torch.int64, "ids"), ids.numel()),
           "ic_index_invalidate")


def ic_index_compact(handle: int, id_map: torch.Tensor) -> int:
    """Drop invalidated rows; ``id_map`` int64 [old size] receives new ids (-1 = dropped).  Returns the new size."""
    n = ctypes.c_int64(-1)
    _check(load_library().ic_index_compact(handle, _dev_ptr(id_map, torch.int64, "id_map"), ctypes.byref(n)),
           "ic_index_compact")
    return n.value


# ---- convenience owner of (arena, handle) -----------------------------------

class Index:
    """Owns the arena tensor and the handle; methods forward to the ABI calls."""

    def __init__(self, d: int, capacity_rows: int, store: int = STORE_BF16, max_queries: int = 64,
                 max_k: int = 64, device="cuda:0"):
        self.d, self.store, self.capacity = d, store, capacity_rows
        self.device = torch.device(device)
        nbytes = ic_workspace_bytes(d, store, capacity_rows, max_queries, max_k)
        if nbytes == 0:
            raise ICError(1, "ic_workspace_bytes")
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        assert self.arena.data_ptr() % IC_ARENA_ALIGN == 0
        self.handle = ic_index_create(d, store, capacity_rows, max_queries, max_k, self.arena)

    def append(self, emb, util=None) -> int:
        return ic_index_append(self.handle, emb, util)

    def search(self, queries, k, lam=0.0, mask=None, out_scores=None, out_ids=None):
        return ic_search(self.handle, queries, k, lam, mask, out_scores, out_ids)

    def __len__(self) -> int:
        return int(load_library().ic_index_size(self.handle))

    def set_timing(self, enable: bool) -> None:
        _check(load_library().ic_index_set_timing(self.handle, int(enable)), "ic_index_set_timing")

    def set_tuning(self, slices: int = 0, list_keys: int = 0) -> None:
        """Launch-shape overrides for tests and sweeps (0 = default); results do not depend on them."""
        _check(load_library().ic_index_set_tuning(self.handle, slices, list_keys), "ic_index_set_tuning")

    def scan_time_ms(self) -> Tuple[float, int]:
        """(summed scan-kernel time in ms, number of launches) since timing was switched on."""
        ms, cnt = ctypes.c_float(0), ctypes.c_int64(0)
        _check(load_library().ic_index_scan_time_ms(self.handle, ctypes.byref(ms), ctypes.byref(cnt)),
               "ic_index_scan_time_ms")
        return float(ms.value), int(cnt.value)

    def tiled_scan_counts(self) -> Tuple[int, int]:
        """(tiles computed a second time, blocks of 64 queries redone) of the last large batch."""
        again, redone = ctypes.c_int64(0), ctypes.c_int64(0)
        _check(load_library().ic_index_tiled_scan_counts(self.handle, ctypes.byref(again), ctypes.byref(redone)),
               "ic_index_tiled_scan_counts")
        return int(again.value), int(redone.value)

    def store_view(self):
        """(rows uint8 [n, row_bytes], scale fp32 [n] | None, util fp32 [n]) as views of the arena."""
        L = load_library()
        rows, stride = ctypes.c_void_p(), ctypes.c_int64()
        scale, util = ctypes.c_void_p(), ctypes.c_void_p()
        _check(L.ic_index_store_view(self.handle, ctypes.byref(rows), ctypes.byref(stride),
                                     ctypes.byref(scale), ctypes.byref(util)), "ic_index_store_view")
        base = self.arena.data_ptr()
        n, rb = len(self), stride.value
        r = self.arena[rows.value - base: rows.value - base + n * rb].view(n, rb)
        u = self.arena[util.value - base: util.value - base + 4 * n].view(torch.float32)
        s = None
        if scale.value:
            s = self.arena[scale.value - base: scale.value - base + 4 * n].view(torch.float32)
        return r, s, u

    def search_threshold(self, queries: torch.Tensor, k: int, min_score: float, lam: float = 0.0,
                         mask: Optional[torch.Tensor] = None):
        return ic_search_threshold(self.handle, queries, k, min_score, lam, mask)

    def self_search(self, first_row: int, count: int, k: int, lam: float = 0.0,
                    mask: Optional[torch.Tensor] = None):
        return ic_self_search(self.handle, first_row, count, k, lam, mask, self.device)

    def search_domains(self, queries: torch.Tensor, k: int, query_domain: torch.Tensor, lam: float = 0.0,
                       mask: Optional[torch.Tensor] = None):
        return ic_search_domains(self.handle, queries, k, query_domain, lam, mask)

    def set_domains(self, ids: torch.Tensor, domains: torch.Tensor) -> None:
        ic_index_set_domains(self.handle, ids, domains)

    def set_utility(self, ids: torch.Tensor, util: torch.Tensor) -> None:
        ic_index_set_utility(self.handle, ids, util)

    def scale_utility(self, factor: float) -> None:
        ic_index_scale_utility(self.handle, factor)

    def invalidate(self, ids: torch.Tensor) -> None:
        ic_index_invalidate(self.handle, ids)

    def compact(self) -> torch.Tensor:
        """Drop invalidated rows; returns the id map (int64 [old size], -1 = dropped)."""
        id_map = torch.empty(max(len(self), 1), dtype=torch.int64, device=self.device)[: len(self)]
        ic_index_compact(self.handle, id_map)
        return id_map

    def close(self) -> None:
        if getattr(self, "handle", None):
            ic_index_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Ivf:
    """Cluster pruning on top of an ``Index``: owns its arena and the handle."""

    def __init__(self, base: Index, K: int, max_probe: int):
        L = load_library()
        self.base, self.K, self.max_probe = base, int(K), int(max_probe)
        nbytes = int(L.ic_ivf_workspace_bytes(base.handle, K, max_probe))
        if nbytes == 0:
            raise ValueError("ic_ivf_workspace_bytes rejected the arguments")
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=base.device)
        h = ctypes.c_void_p()
        _check(L.ic_ivf_create(ctypes.byref(h), base.handle, K, max_probe, self.arena.data_ptr(), nbytes),
               "ic_ivf_create")
        self.handle = h.value

    def set_centroids(self, centroids: torch.Tensor) -> None:
        assert centroids.shape == (self.K, self.base.d)
        _check(load_library().ic_ivf_set_centroids(self.handle, _dev_ptr(centroids, torch.float32, "centroids")),
               "ic_ivf_set_centroids")

    def assign(self) -> None:
        _check(load_library().ic_ivf_assign(self.handle), "ic_ivf_assign")

    def set_assignment(self, assign: torch.Tensor) -> None:
        assert assign.numel() == len(self.base)
        _check(load_library().ic_ivf_set_assignment(self.handle, _dev_ptr(assign, torch.int32, "assign")),
               "ic_ivf_set_assignment")

    def update_centroids(self) -> None:
        _check(load_library().ic_ivf_update_centroids(self.handle), "ic_ivf_update_centroids")

    def train(self, iters: int) -> None:
        _check(load_library().ic_ivf_train(self.handle, iters), "ic_ivf_train")

    def search(self, queries: torch.Tensor, k: int, nprobe: int, lam: float = 0.0):
        Q = queries.shape[0]
        out_scores = torch.empty((Q, k), dtype=torch.float32, device=queries.device)
        out_ids = torch.empty((Q, k), dtype=torch.int64, device=queries.device)
        _check(load_library().ic_ivf_search(self.handle, _dev_ptr(queries, torch.float32, "queries"), Q, k, nprobe,
                                            float(lam), out_scores.data_ptr(), out_ids.data_ptr()), "ic_ivf_search")
        return out_scores, out_ids

    def probed_clusters(self, queries: torch.Tensor, nprobe: int) -> torch.Tensor:
        """The nprobe nearest centroids of every query (int64 [Q, nprobe]): the same ``ic_search`` on the
        centroid index that ``ic_ivf_search`` starts with."""
        L = load_library()
        c = ctypes.c_void_p()
        _check(L.ic_ivf_view(self.handle, None, None, None, ctypes.byref(c), None), "ic_ivf_view")
        return ic_search(c.value, queries, nprobe)[1]

    def view(self):
        """(assign int32 [size], offsets int64 [K+1], perm int32 [listed rows], centroid rows uint8 [K, row_bytes],
        centroid scales | None) as views of the arena."""
        L = load_library()
        a, o, p, c, s = (ctypes.c_void_p() for _ in range(5))
        _check(L.ic_ivf_view(self.handle, ctypes.byref(a), ctypes.byref(o), ctypes.byref(p), ctypes.byref(c),
                             ctypes.byref(s)), "ic_ivf_view")
        base = self.arena.data_ptr()
        n = len(self.base)
        assign = self.arena[a.value - base: a.value - base + 4 * n].view(torch.int32)
        offsets = self.arena[o.value - base: o.value - base + 8 * (self.K + 1)].view(torch.int64)
        listed = int(L.ic_index_size(s.value))
        perm = self.arena[p.value - base: p.value - base + 4 * listed].view(torch.int32)
        rows, stride = ctypes.c_void_p(), ctypes.c_int64()
        scale = ctypes.c_void_p()
        _check(L.ic_index_store_view(c.value, ctypes.byref(rows), ctypes.byref(stride), ctypes.byref(scale), None),
               "ic_index_store_view")
        rb = stride.value
        crow = self.arena[rows.value - base: rows.value - base + self.K * rb].view(self.K, rb)
        cscale = None
        if scale.value:
            cscale = self.arena[scale.value - base: scale.value - base + 4 * self.K].view(torch.float32)
        return assign, offsets, perm, crow, cscale

    def close(self) -> None:
        if getattr(self, "handle", None):
            _check(load_library().ic_ivf_destroy(self.handle), "ic_ivf_destroy")
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
