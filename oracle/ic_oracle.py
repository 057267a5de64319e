"""ctypes access to the CPU reference (``ic_oracle.c``) plus a NumPy restatement.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module,
and this module never imports the product package.

The reference states IC-Cache's stage-1 example selection (Sec. 4.1, and the
GetSimilarExamples step of Algorithm 1) as exact brute force in fp64:
cosine similarity of the request embedding with every cached example
embedding, plus ``lambda * utility`` and a validity mask (what the Example
Manager of Sec. 4.3 keeps per example), best ``k`` under the total order
(score descending, index ascending).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ic_oracle.c")
_LIB = os.path.join(_HERE, "libic_oracle.so")

_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_u8p = ctypes.POINTER(ctypes.c_uint8)
_u16p = ctypes.POINTER(ctypes.c_uint16)
_i64p = ctypes.POINTER(ctypes.c_int64)


def build(force: bool = False) -> str:
    """Compile ``ic_oracle.c`` with gcc (OpenMP) into ``libic_oracle.so``."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", _SRC, "-o", _LIB, "-lm"]
        )
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.ico_num_threads.restype = ctypes.c_int
        L.ico_begin.restype = ctypes.c_void_p
        L.ico_begin.argtypes = [_f32p, _f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                                ctypes.c_float, ctypes.c_int]
        L.ico_scan.restype = ctypes.c_int
        L.ico_scan.argtypes = [ctypes.c_void_p, _f32p, _f32p, _u8p, _f32p, ctypes.c_int64,
                               ctypes.c_int64]
        L.ico_finish.restype = ctypes.c_int
        L.ico_finish.argtypes = [ctypes.c_void_p, _f32p, _i64p, _f64p]
        L.ico_free.restype = None
        L.ico_free.argtypes = [ctypes.c_void_p]
        L.ico_scores.restype = ctypes.c_int
        L.ico_scores.argtypes = [_f32p, _f32p, _f32p, ctypes.c_int64, ctypes.c_int32, _f32p, _f32p,
                                 ctypes.c_int64, ctypes.c_float, ctypes.c_int, _f64p]
        L.ico_quantize_bf16.restype = ctypes.c_int
        L.ico_quantize_bf16.argtypes = [_f32p, ctypes.c_int64, ctypes.c_int32, _u16p]
        L.ico_quantize_fp8.restype = ctypes.c_int
        L.ico_quantize_fp8.argtypes = [_f32p, ctypes.c_int64, ctypes.c_int32, _u8p, _f32p]
        L.ico_decode_bf16.restype = ctypes.c_int
        L.ico_decode_bf16.argtypes = [_u16p, ctypes.c_int64, _f32p]
        L.ico_decode_e4m3.restype = ctypes.c_int
        L.ico_decode_e4m3.argtypes = [_u8p, ctypes.c_int64, _f32p]
        L.ico_encode_e4m3.restype = ctypes.c_int
        L.ico_encode_e4m3.argtypes = [_f32p, ctypes.c_int64, _u8p]
        L.ico_encode_bf16.restype = ctypes.c_int
        L.ico_encode_bf16.argtypes = [_f32p, ctypes.c_int64, _u16p]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().ico_num_threads())


def _f32(a, shape_len: int) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    assert a.ndim == shape_len, a.shape
    return a


def _ptr(a: Optional[np.ndarray], typ):
    return None if a is None else a.ctypes.data_as(typ)


class Scan:
    """Chunked brute-force search: feed the cache in row blocks, then ``finish``.

    ``normalize=True`` is the definition (true cosine).  ``normalize=False``
    takes the rows and queries as already unit length and forms the plain inner
    product, times optional per-row / per-query scales; this is how the values a
    quantised store holds are fed through the same search.
    """

    def __init__(self, queries, k: int, lam: float = 0.0, normalize: bool = True,
                 q_scale=None):
        self.Qm = _f32(queries, 2)
        self.Q, self.d = self.Qm.shape
        self.k = int(k)
        self.q_scale = None if q_scale is None else _f32(q_scale, 1)
        if self.q_scale is not None:
            assert self.q_scale.shape[0] == self.Q
        self._st = lib().ico_begin(_ptr(self.Qm, _f32p), _ptr(self.q_scale, _f32p), self.Q,
                                   self.d, self.k, float(lam), int(bool(normalize)))
        if not self._st:
            raise ValueError("ico_begin rejected its arguments")
        self._next = 0

    def scan(self, E, U=None, mask=None, row_scale=None, base_id: Optional[int] = None) -> None:
        E = _f32(E, 2)
        n = E.shape[0]
        assert E.shape[1] == self.d
        U = None if U is None else _f32(U, 1)
        row_scale = None if row_scale is None else _f32(row_scale, 1)
        if mask is not None:
            mask = np.ascontiguousarray(mask, dtype=np.uint8)
            assert mask.shape == (n,)
        if U is not None:
            assert U.shape == (n,)
        if row_scale is not None:
            assert row_scale.shape == (n,)
        base = self._next if base_id is None else int(base_id)
        rc = lib().ico_scan(self._st, _ptr(E, _f32p), _ptr(U, _f32p), _ptr(mask, _u8p),
                            _ptr(row_scale, _f32p), n, base)
        if rc != 0:
            raise RuntimeError(f"ico_scan failed ({rc})")
        self._next = base + n

    def finish(self) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        """Return (scores fp32 [Q,k], ids int64 [Q,k], scores fp64 [Q,k])."""
        s = np.empty((self.Q, self.k), dtype=np.float32)
        i = np.empty((self.Q, self.k), dtype=np.int64)
        s64 = np.empty((self.Q, self.k), dtype=np.float64)
        rc = lib().ico_finish(self._st, _ptr(s, _f32p), _ptr(i, _i64p), _ptr(s64, _f64p))
        if rc != 0:
            raise RuntimeError(f"ico_finish failed ({rc})")
        return s, i, s64

    def close(self) -> None:
        if self._st:
            lib().ico_free(self._st)
            self._st = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def search(E, queries, k: int, lam: float = 0.0, U=None, mask=None, normalize: bool = True,
           row_scale=None, q_scale=None):
    """Exact top-k of ``cos + lam*U`` over the valid rows.  Returns (s32, ids, s64)."""
    sc = Scan(queries, k, lam, normalize, q_scale)
    sc.scan(E, U, mask, row_scale)
    out = sc.finish()
    sc.close()
    return out


def scores(E, queries, lam: float = 0.0, U=None, normalize: bool = True, row_scale=None,
           q_scale=None) -> np.ndarray:
    """Dense fp64 score matrix [Q,N], same arithmetic as ``search`` (no mask)."""
    E = _f32(E, 2)
    Qm = _f32(queries, 2)
    U = None if U is None else _f32(U, 1)
    row_scale = None if row_scale is None else _f32(row_scale, 1)
    q_scale = None if q_scale is None else _f32(q_scale, 1)
    out = np.empty((Qm.shape[0], E.shape[0]), dtype=np.float64)
    rc = lib().ico_scores(_ptr(E, _f32p), _ptr(U, _f32p), _ptr(row_scale, _f32p), E.shape[0],
                          E.shape[1], _ptr(Qm, _f32p), _ptr(q_scale, _f32p), Qm.shape[0],
                          float(lam), int(bool(normalize)), _ptr(out, _f64p))
    if rc != 0:
        raise RuntimeError(f"ico_scores failed ({rc})")
    return out


# --------------------------------------------------------------------------
# store formats (independent CPU statement)
# --------------------------------------------------------------------------

def quantize_bf16(X) -> np.ndarray:
    """uint16 bf16 codes [n,d] of the unit-normalised rows (round to nearest even)."""
    X = _f32(X, 2)
    out = np.empty(X.shape, dtype=np.uint16)
    rc = lib().ico_quantize_bf16(_ptr(X, _f32p), X.shape[0], X.shape[1], _ptr(out, _u16p))
    assert rc == 0
    return out


def quantize_fp8(X) -> Tuple[np.ndarray, np.ndarray]:
    """(uint8 E4M3 codes [n,d], fp32 scale [n]) of the unit-normalised rows."""
    X = _f32(X, 2)
    codes = np.empty(X.shape, dtype=np.uint8)
    scale = np.empty((X.shape[0],), dtype=np.float32)
    rc = lib().ico_quantize_fp8(_ptr(X, _f32p), X.shape[0], X.shape[1], _ptr(codes, _u8p),
                                _ptr(scale, _f32p))
    assert rc == 0
    return codes, scale


def decode_bf16(codes) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint16)
    out = np.empty(codes.shape, dtype=np.float32)
    assert lib().ico_decode_bf16(_ptr(codes, _u16p), codes.size, _ptr(out, _f32p)) == 0
    return out


def decode_e4m3(codes) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    out = np.empty(codes.shape, dtype=np.float32)
    assert lib().ico_decode_e4m3(_ptr(codes, _u8p), codes.size, _ptr(out, _f32p)) == 0
    return out


def encode_e4m3(x) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint8)
    assert lib().ico_encode_e4m3(_ptr(x, _f32p), x.size, _ptr(out, _u8p)) == 0
    return out


def encode_bf16(x) -> np.ndarray:
    """Raw bf16 codes of fp32 values as given (no normalisation): round to nearest, ties to even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    assert lib().ico_encode_bf16(_ptr(x, _f32p), x.size, _ptr(out, _u16p)) == 0
    return out


# --------------------------------------------------------------------------
# NumPy restatement, for tiny inputs only (checks the C reference)
# --------------------------------------------------------------------------

def search_numpy(E, queries, k: int, lam: float = 0.0, U=None, mask=None):
    """Same definition through NumPy float64 and a full lexicographic sort."""
    E = np.asarray(E, dtype=np.float64)
    Qm = np.asarray(queries, dtype=np.float64)
    N = E.shape[0]
    en = np.sqrt((E * E).sum(axis=1))
    qn = np.sqrt((Qm * Qm).sum(axis=1))
    den = qn[:, None] * en[None, :]
    dot = Qm @ E.T
    cos = np.where(den > 0, dot / np.where(den > 0, den, 1.0), 0.0)
    s = cos + (0.0 if U is None else float(np.float32(lam)) * np.asarray(U, dtype=np.float64)[None, :])
    valid = np.ones(N, dtype=bool) if mask is None else (np.asarray(mask) != 0)
    ids_all = np.arange(N, dtype=np.int64)
    out_s = np.full((Qm.shape[0], k), -np.inf, dtype=np.float64)
    out_i = np.full((Qm.shape[0], k), -1, dtype=np.int64)
    for q in range(Qm.shape[0]):
        cand = ids_all[valid]
        order = np.lexsort((cand, -s[q, cand]))[:k]
        out_s[q, :len(order)] = s[q, cand[order]]
        out_i[q, :len(order)] = cand[order]
    return out_s.astype(np.float32), out_i, out_s


# --------------------------------------------------------------------------
# Store maintenance (Example Manager, Sec. 4.3 "Capping Example Cache Size over Time"): what
# the store holds after utilities are refreshed or decayed and after evicted examples are
# squeezed out.  Plain definitions on host arrays.
# --------------------------------------------------------------------------

def set_utility(U, ids, values):
    """U with U[ids[j]] = values[j]; ids outside the store are ignored (ids must be distinct)."""
    out = np.array(U, dtype=np.float32, copy=True)
    for j, i in enumerate(np.asarray(ids, dtype=np.int64)):
        if 0 <= i < out.shape[0]:
            out[i] = np.float32(values[j])
    return out


def scale_utility(U, factor):
    """Every utility times ``factor``, one fp32 multiplication each (the hourly decay uses 0.9)."""
    return (np.asarray(U, dtype=np.float32) * np.float32(factor)).astype(np.float32)


def invalidate(valid, ids):
    """Validity flags after the rows ``ids`` were evicted."""
    out = np.array(valid, dtype=np.uint8, copy=True)
    for i in np.asarray(ids, dtype=np.int64):
        if 0 <= i < out.shape[0]:
            out[i] = 0
    return out


def compaction_map(valid):
    """New id of every row once the invalid rows are dropped and the others keep their order:
    the number of valid rows before it, or -1 for a dropped row.  Returns (id_map, new_size)."""
    out = np.full(len(valid), -1, dtype=np.int64)
    nxt = 0
    for i, v in enumerate(valid):
        if v:
            out[i] = nxt
            nxt += 1
    return out, nxt


# --------------------------------------------------------------------------
# Threshold mode (Sec. 4.1, "Selecting Example Combinations"): examples below a score threshold
# are dropped, so the number selected varies per query.
# --------------------------------------------------------------------------

def search_threshold(E, queries, k: int, min_score: float, lam: float = 0.0, U=None, mask=None):
    """search(), then entries with fp64 score < min_score become (-inf, -1).
    Returns (scores fp32, ids, scores fp64, counts)."""
    s32, ids, s64 = search(E, queries, k, lam, U, mask)
    s32, ids, s64 = s32.copy(), ids.copy(), s64.copy()
    drop = (ids < 0) | (s64 < float(min_score))
    s32[drop] = -np.inf
    s64[drop] = -np.inf
    ids[drop] = -1
    return s32, ids, s64, (~drop).sum(axis=1).astype(np.int32)


# --------------------------------------------------------------------------
# Sharing domains (Sec. 4.3, "How Does IC-Cache Respect Privacy?": cached data is shared only
# within designated user domains).  A row of domain 0 is shared with everyone; any other row is
# seen only by queries of its own domain.
# --------------------------------------------------------------------------

def search_domains(E, queries, k: int, row_domain, query_domain, lam: float = 0.0, U=None, mask=None,
                   normalize: bool = True, row_scale=None, q_scale=None):
    """One query at a time: search() with the rows the query may not see masked out."""
    E = np.asarray(E)
    queries = np.asarray(queries)
    row_domain = np.asarray(row_domain, dtype=np.int64)
    query_domain = np.asarray(query_domain, dtype=np.int64)
    n = E.shape[0]
    base = np.ones(n, dtype=bool) if mask is None else (np.asarray(mask) != 0)
    out = []
    for j in range(queries.shape[0]):
        visible = base & ((row_domain == 0) | (row_domain == query_domain[j]))
        qs = None if q_scale is None else np.asarray(q_scale)[j:j + 1]
        out.append(search(E, queries[j:j + 1], k, lam, U, visible.astype(np.uint8), normalize, row_scale, qs))
    return tuple(np.concatenate([o[t] for o in out], axis=0) for t in range(3))


# --------------------------------------------------------------------------
# Self-search (Sec. 2.3, "Voluminous requests lead to pervasive similarity": the top-1 similarity of
# every request to the others): the queries are rows of the cache itself, each left out of its
# own result.
# --------------------------------------------------------------------------

def self_search(E, first_row: int, count: int, k: int, lam: float = 0.0, U=None, mask=None):
    """For each row r in [first_row, first_row + count): the best k of the valid rows other than r.
    Stated through search(): the best k + 1 over all valid rows with r removed (or, when r is not
    among them, with the last one removed)."""
    E = np.asarray(E, dtype=np.float32)
    rows = np.arange(first_row, first_row + count)
    s32, ids, s64 = search(E, E[rows], k + 1, lam, U, mask)
    out32 = np.full((count, k), -np.inf, dtype=np.float32)
    out64 = np.full((count, k), -np.inf, dtype=np.float64)
    outi = np.full((count, k), -1, dtype=np.int64)
    for j, r in enumerate(rows):
        keep = [p for p in range(k + 1) if ids[j, p] != r][:k]
        outi[j, :len(keep)] = ids[j, keep]
        out32[j, :len(keep)] = s32[j, keep]
        out64[j, :len(keep)] = s64[j, keep]
    return out32, outi, out64


# --------------------------------------------------------------------------
# Cluster pruning (Sec. 4.1, "Two-Stage Scalable Example Selection"): K-Means clusters offline;
# online the nearest centroids first, then only the examples of those clusters.  Each step is
# written out plainly in fp64; search() above serves as the "nearest" primitive.
# --------------------------------------------------------------------------

def _unit(X):
    X = np.asarray(X, dtype=np.float64)
    nrm = np.sqrt((X * X).sum(axis=1, keepdims=True))
    return np.where(nrm > 0, X / np.where(nrm > 0, nrm, 1.0), 0.0)


def ivf_assign(E, C):
    """Cluster of every row: the centroid with the highest cosine, lowest centroid id on ties."""
    _, ids, _ = search(np.asarray(C, dtype=np.float32), np.asarray(E, dtype=np.float32), 1)
    return ids[:, 0].astype(np.int32)


def ivf_lists(assign, K: int, valid=None):
    """offsets [K + 1] and, per cluster, the ascending ids of its rows (rows with a cluster outside
    [0, K) or valid == 0 are in no list)."""
    assign = np.asarray(assign)
    ok = (assign >= 0) & (assign < K)
    if valid is not None:
        ok &= np.asarray(valid) != 0
    lists = [np.flatnonzero(ok & (assign == c)).astype(np.int64) for c in range(K)]
    offsets = np.zeros(K + 1, dtype=np.int64)
    offsets[1:] = np.cumsum([len(x) for x in lists])
    return offsets, lists


def ivf_update(E, assign, K: int, C_old, valid=None, normalize: bool = True):
    """K-Means update on the unit sphere: every centroid becomes the normalised sum of the unit
    rows of its list; an empty list keeps its (normalised) centroid.  fp64.  ``normalize=False``
    takes the rows as they are (this is how the values a quantised store holds are fed through
    the same step, as in search())."""
    Eu = _unit(E) if normalize else np.asarray(E, dtype=np.float64)
    out = _unit(C_old).copy()
    _, lists = ivf_lists(assign, K, valid)
    for c, ids in enumerate(lists):
        if len(ids):
            out[c] = _unit(Eu[ids].sum(axis=0, keepdims=True))[0]
    return out


def ivf_kmeans(E, K: int, iters: int):
    """K-Means as the library runs it: start from the rows at positions floor(c * N / K), then
    ``iters`` times (assign, update), then a final assign.  Returns (centroids fp64, assign)."""
    E = np.asarray(E, dtype=np.float32)
    N = E.shape[0]
    C = _unit(E[[(c * N) // K for c in range(K)]])
    for _ in range(iters):
        C = ivf_update(E, ivf_assign(E, C), K, C)
    return C, ivf_assign(E, C)


def ivf_search(E, C, assign, queries, k: int, nprobe: int, lam: float = 0.0, U=None, valid=None):
    """Top-k over the rows of the nprobe nearest clusters of each query.
    Returns (scores fp32, ids, scores fp64, probes [Q, nprobe])."""
    E = np.asarray(E, dtype=np.float32)
    Qm = np.asarray(queries, dtype=np.float32)
    K = np.asarray(C).shape[0]
    _, probes, _ = search(np.asarray(C, dtype=np.float32), Qm, nprobe)
    _, lists = ivf_lists(assign, K, valid)
    Q = Qm.shape[0]
    s32 = np.full((Q, k), -np.inf, dtype=np.float32)
    s64 = np.full((Q, k), -np.inf, dtype=np.float64)
    ids = np.full((Q, k), -1, dtype=np.int64)
    for q in range(Q):
        cand = np.concatenate([lists[c] for c in probes[q] if c >= 0] + [np.zeros(0, np.int64)])
        if not len(cand):
            continue
        cand.sort()
        a32, ai, a64 = search(E[cand], Qm[q:q + 1], k, lam, None if U is None else np.asarray(U)[cand])
        m = int((ai[0] >= 0).sum())
        ids[q, :m] = cand[ai[0, :m]]
        s32[q, :m] = a32[0, :m]
        s64[q, :m] = a64[0, :m]
    return s32, ids, s64, probes
