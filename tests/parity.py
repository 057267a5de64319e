"""Comparison rules between a top-k result and the CPU reference.

Two checks, both phrased with reference values only:

* **band** (against the fp32-master reference, tolerance ``tau`` = 2e-2 for a
  bf16 store, 6e-2 for fp8): with ``s*`` the reference scores and ``s*_(r)`` the
  r-th best, every example with ``s* >= s*_(k+1) + tau`` must be returned, every
  returned example must have ``s* > s*_(k) - tau``, and every returned score must
  be within ``tau`` of ``s*``.  When the k-th and (k+1)-th reference scores are
  at least ``tau`` apart this is set equality.

* **sharp** (against the reference fed with the values the store holds, from
  the reference's own quantiser; ``tau_q`` = 1e-4 covers fp32 accumulation
  order for scores of order 1; a case with a large ``lambda * utility`` passes
  the same bound scaled to the fp32 spacing at that magnitude): over a candidate pool (all rows, or the returned ids plus the
  reference's top-K'), returned scores match within ``tau_q`` and the returned
  set equals the pool's top-k except for members within ``tau_q`` of the k-th.

Structure is always checked: count = min(k, valid rows), ids distinct and
valid, rows sorted by (score desc, id asc), tail padded with (-inf, -1).
"""
from __future__ import annotations

from typing import Callable, Optional

import numpy as np

from oracle import ic_oracle as orc

TAU = {"bf16": 2e-2, "fp8": 6e-2}
TAU_Q = 1e-4


def quantised_scores(store: str, E: np.ndarray, U: Optional[np.ndarray], Qm: np.ndarray,
                     lam: float) -> np.ndarray:
    """fp64 scores [Q, n] of the values a ``store``-format index holds for rows E."""
    if E.shape[0] == 0:
        return np.zeros((Qm.shape[0], 0))
    if store == "bf16":
        e = orc.decode_bf16(orc.quantize_bf16(E))
        q = orc.decode_bf16(orc.quantize_bf16(Qm))
        return orc.scores(e, q, lam=lam, U=U, normalize=False)
    ce, se = orc.quantize_fp8(E)
    cq, sq = orc.quantize_fp8(Qm)
    return orc.scores(orc.decode_e4m3(ce), orc.decode_e4m3(cq), lam=lam, U=U, normalize=False,
                      row_scale=se, q_scale=sq)


def check_structure(gs: np.ndarray, gi: np.ndarray, n_valid: int, k: int,
                    is_valid: Callable[[np.ndarray], np.ndarray], where: str) -> int:
    m = min(k, n_valid)
    assert np.all(gi[m:] == -1) and np.all(np.isneginf(gs[m:])), f"{where}: padding tail"
    ids = gi[:m]
    assert np.all(ids >= 0), f"{where}: too few results ({ids})"
    assert len(set(ids.tolist())) == m, f"{where}: duplicate ids"
    assert np.all(is_valid(ids)), f"{where}: invalid row returned"
    s = gs[:m]
    assert np.all(np.isfinite(s)), f"{where}: non-finite score"
    ds = np.diff(s)
    assert np.all(ds <= 0), f"{where}: scores not sorted"
    tie = ds == 0
    assert np.all(np.diff(ids)[tie] > 0), f"{where}: equal scores not in id order"
    return m


def check_query(store: str, gs: np.ndarray, gi: np.ndarray, k: int, lam: float,
                q_vec: np.ndarray, ref_ids: np.ndarray, ref_s64: np.ndarray, n_valid: int,
                fetch: Callable[[np.ndarray], tuple], is_valid: Callable[[np.ndarray], np.ndarray],
                where: str, sharp: bool = True, tau_q: float = TAU_Q) -> dict:
    """Check one query.  ``ref_*`` is the reference's best-K' list (K' >= min(k+1, n_valid))
    on the fp32 masters; ``fetch(ids)`` returns (E rows fp32, U or None) for given ids."""
    tau = TAU[store]
    m = check_structure(gs, gi, n_valid, k, is_valid, where)
    ret = gi[:m]
    ref_n = int((ref_ids >= 0).sum())
    assert ref_n >= min(k + 1, n_valid), f"{where}: reference list too short"
    stats = {"recall": 1.0, "max_err": 0.0, "max_err_q": 0.0}
    if m == 0:
        return stats

    # ---- band check on the fp32 masters
    E_ret, U_ret = fetch(ret)
    s_star = orc.scores(E_ret, q_vec[None], lam=lam, U=U_ret)[0]
    err = np.abs(gs[:m].astype(np.float64) - s_star)
    stats["max_err"] = float(err.max())
    assert err.max() <= tau, f"{where}: score off by {err.max():.3e} > {tau}"
    s_k = ref_s64[m - 1]
    assert np.all(s_star > s_k - tau), f"{where}: returned example below the band"
    if ref_n > k:
        must = ref_ids[:k][ref_s64[:k] >= ref_s64[k] + tau]
        missing = np.setdiff1d(must, ret)
        assert missing.size == 0, f"{where}: must-return examples missing: {missing[:8]}"
    stats["recall"] = float(np.isin(ref_ids[:m], ret).mean())

    # ---- sharp check on the stored values
    if sharp:
        pool = np.union1d(ret, ref_ids[:ref_n])
        E_pool, U_pool = fetch(pool)
        s_hat = quantised_scores(store, E_pool, U_pool, q_vec[None], lam)[0]
        pos = {int(i): j for j, i in enumerate(pool)}
        s_ret = np.array([s_hat[pos[int(i)]] for i in ret])
        err_q = np.abs(gs[:m].astype(np.float64) - s_ret)
        stats["max_err_q"] = float(err_q.max())
        assert err_q.max() <= tau_q, f"{where}: stored-value score off by {err_q.max():.3e}"
        order = np.lexsort((pool, -s_hat))
        top = pool[order][:m]
        kth = s_hat[order][m - 1]
        extra = np.setdiff1d(ret, top)       # returned but not in the pool's top-m
        lost = np.setdiff1d(top, ret)        # in the pool's top-m but not returned
        for i in extra:
            assert s_hat[pos[int(i)]] > kth - tau_q, f"{where}: id {i} returned from below the cut"
        for i in lost:
            assert s_hat[pos[int(i)]] < kth + tau_q, f"{where}: id {i} (score above the cut) missing"
    return stats


def check_batch(store: str, gpu_scores: np.ndarray, gpu_ids: np.ndarray, E: np.ndarray,
                U: Optional[np.ndarray], mask: Optional[np.ndarray], Qm: np.ndarray, k: int,
                lam: float, where: str, queries=None, sharp: bool = True, tau_q: float = TAU_Q) -> dict:
    """Whole-cache check for host-resident masters (small and medium sizes)."""
    N = E.shape[0]
    valid = np.ones(N, bool) if mask is None else (mask != 0)
    n_valid = int(valid.sum())
    qs = range(Qm.shape[0]) if queries is None else queries
    qs = list(qs)
    kk = min(max(4 * k, k + 1), max(N, 1))
    _, ref_i, ref_s = orc.search(E, Qm[qs], k=kk, lam=lam, U=U, mask=mask)

    def fetch(ids):
        return E[ids], (None if U is None else U[ids])

    agg = {"recall": [], "max_err": 0.0, "max_err_q": 0.0}
    for j, q in enumerate(qs):
        st = check_query(store, gpu_scores[q], gpu_ids[q], k, lam, Qm[q], ref_i[j], ref_s[j], n_valid,
                         fetch, lambda ids: valid[ids], f"{where} q={q}", sharp=sharp, tau_q=tau_q)
        agg["recall"].append(st["recall"])
        agg["max_err"] = max(agg["max_err"], st["max_err"])
        agg["max_err_q"] = max(agg["max_err_q"], st["max_err_q"])
    agg["recall"] = float(np.mean(agg["recall"])) if agg["recall"] else 1.0
    return agg
