"""GPU parity of access-controlled search (per-row sharing domains, one domain per query), through
the C ABI: no row of a foreign domain is ever returned (exact), and each query's result is within
the comparison band of the CPU reference over the rows that query may see."""
import sys

import numpy as np
import pytest
import torch

import parity
import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def pkg():
    import paper_2501_12689_amd as p
    p.load_library()
    return p


def _domains(N, Q, seed, tiny_rows=5):
    """Half of the rows shared (0), the rest spread over domains 1..4, and a domain 9 with only
    `tiny_rows` rows; queries drawn from 0..4, 9 and 7 (a domain without rows)."""
    rng = np.random.default_rng(seed)
    dom = np.where(rng.random(N) < 0.5, 0, rng.integers(1, 5, N)).astype(np.int32)
    dom[rng.choice(N, tiny_rows, replace=False)] = 9
    qd = rng.choice(np.array([0, 1, 2, 3, 4, 9, 7], dtype=np.int32), Q)
    if Q >= 7:
        qd[:7] = [0, 1, 2, 3, 4, 9, 7]
    return dom, qd.astype(np.int32)


def _check(store, gs, gi, E, U, M, Qm, k, lam, dom, qd, where, per_domain=6):
    N = E.shape[0]
    # exact: nothing outside the query's view, nothing masked
    ok = gi >= 0
    rows = np.where(ok, gi, 0)
    foreign = ok & (dom[rows] != 0) & (dom[rows] != qd[:, None])
    assert not foreign.any(), f"{where}: {int(foreign.sum())} rows of foreign domains returned"
    base = np.ones(N, bool) if M is None else (M != 0)
    worst = {"max_err": 0.0, "recall": 1.0}
    for D in np.unique(qd):
        vis = (base & ((dom == 0) | (dom == D))).astype(np.uint8)
        qs = np.flatnonzero(qd == D)
        qs = qs[:: max(1, len(qs) // per_domain)]
        st = parity.check_batch(store, gs, gi, E, U, vis, Qm, k, lam, f"{where} domain={D}", queries=qs.tolist())
        worst["max_err"] = max(worst["max_err"], st["max_err"])
        worst["recall"] = min(worst["recall"], st["recall"])
    return worst


CASES = [
    # store, N, d, Q, max_q, k, lam, util, p_valid
    ("bf16", 40000, 96, 7, 8, 10, 0.0, "none", 1.0),            # streaming scan, no pilot
    ("bf16", 290000, 128, 60, 64, 32, 0.3, "uniform", 0.9),     # streaming scan with the pilot
    ("fp8", 70000, 128, 150, 64, 16, 0.2, "beta25", 0.95),      # query chunks of 64: domains follow the chunk
    ("bf16", 300000, 128, 300, 300, 16, 0.2, "beta25", 0.95),   # tiled scan
    ("fp8", 280000, 256, 260, 260, 40, 0.0, "none", 1.0),       # tiled scan, fp8
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "-".join(str(x) for x in c))
def test_search_domains(pkg, oracle, case):
    store, N, d, Q, max_q, k, lam, util, pv = case
    print(f"[case] search_domains {case}", flush=True)
    sys.stdout.flush()
    cfg = workloads.Config("D", N=N, d=d, clusters=32, Q=Q, k=k, store=store, zipf=1.1, lam=lam, util=util,
                           p_valid=pv, seed=9700 + CASES.index(case))
    wl = workloads.Workload(cfg, "cpu")
    E, U, M = wl.rows(0, N)
    Qm = wl.queries()
    dom, qd = _domains(N, Q, cfg.seed)
    sid = pkg.STORE_BF16 if store == "bf16" else pkg.STORE_FP8_E4M3
    ix = pkg.Index(d, N, sid, max_q, k, DEV)
    ix.append(E.to(DEV), None if U is None else U.to(DEV))
    md = None if M is None else M.to(DEV)
    qdev = Qm.to(DEV)
    # before any domain is set every row is shared: the plain result, bit for bit
    s0, i0 = ix.search(qdev, k, lam, md)
    s1, i1 = ix.search_domains(qdev, k, torch.from_numpy(qd).to(DEV), lam, md)
    torch.cuda.synchronize()
    assert torch.equal(i0, i1) and torch.equal(s0, s1)
    ix.set_domains(torch.arange(N, device=DEV), torch.from_numpy(dom).to(DEV))
    s, i = ix.search_domains(qdev, k, torch.from_numpy(qd).to(DEV), lam, md)
    torch.cuda.synchronize()
    En, Un, Mn = E.numpy(), (None if U is None else U.numpy()), (None if M is None else M.numpy())
    st = _check(store, s.cpu().numpy(), i.cpu().numpy(), En, Un, Mn, Qm.numpy(), k, lam, dom, qd, str(case))
    # the reference's own entry point on a few queries, ids outside the band must agree exactly
    pick = list(range(0, Q, max(1, Q // 5)))
    r32, ri, r64 = oracle.search_domains(En, Qm.numpy()[pick], k + 1, dom, qd[pick], lam, Un, Mn)
    gi = i.cpu().numpy()
    tau = parity.TAU[store]
    for t, q in enumerate(pick):
        kth1 = r64[t, k] if ri[t, k] >= 0 else -np.inf
        sure = ri[t, :k][(r64[t, :k] >= kth1 + tau) & (ri[t, :k] >= 0)]
        assert set(sure.tolist()) <= set(gi[q].tolist()), f"{case} q={q}"
        assert (gi[q] >= 0).sum() == (ri[t, :k] >= 0).sum()
    # plain searches ignore the domains
    s2, i2 = ix.search(qdev, k, lam, md)
    torch.cuda.synchronize()
    assert torch.equal(i0, i2) and torch.equal(s0, s2)
    print(f"   recall {st['recall']:.4f} max_err {st['max_err']:.2e}", flush=True)
    ix.close()


def test_domains_follow_rows_through_compaction(pkg, oracle):
    print("[case] domains through compaction", flush=True)
    sys.stdout.flush()
    N, d, Q, k, lam = 50000, 64, 40, 12, 0.25
    cfg = workloads.Config("D", N=N, d=d, clusters=16, Q=Q, k=k, store="bf16", zipf=1.1, lam=lam, util="uniform",
                           p_valid=1.0, seed=9790)
    wl = workloads.Workload(cfg, "cpu")
    E, U, _ = wl.rows(0, N)
    Qm = wl.queries()
    dom, qd = _domains(N, Q, 9790, tiny_rows=30)
    ix = pkg.Index(d, N, pkg.STORE_BF16, Q, k, DEV)
    ix.append(E.to(DEV), U.to(DEV))
    ix.set_domains(torch.arange(N, device=DEV), torch.from_numpy(dom).to(DEV))
    rng = np.random.default_rng(5)
    gone = np.sort(rng.choice(N, N // 3, replace=False))
    ix.invalidate(torch.from_numpy(gone).to(DEV))
    id_map = ix.compact()
    n_new = len(ix)
    torch.cuda.synchronize()
    keep = np.setdiff1d(np.arange(N), gone)
    assert n_new == len(keep)
    assert np.array_equal(id_map.cpu().numpy(), oracle.compaction_map(np.isin(np.arange(N), keep).astype(np.uint8))[0])
    s, i = ix.search_domains(Qm.to(DEV), k, torch.from_numpy(qd).to(DEV), lam)
    torch.cuda.synchronize()
    _check("bf16", s.cpu().numpy(), i.cpu().numpy(), E.numpy()[keep], U.numpy()[keep], None, Qm.numpy(), k, lam,
           dom[keep], qd, "after compaction")
    # rows appended afterwards are shared
    E2 = wl.rows(N, 1000)[0]
    first = ix.append(E2.to(DEV), None)
    assert first == n_new
    s, i = ix.search_domains(E2[:8].to(DEV), 1, torch.full((8,), 7, dtype=torch.int32, device=DEV), 0.0)
    torch.cuda.synchronize()
    assert i[:, 0].cpu().tolist() == list(range(first, first + 8))
    ix.close()


def test_domain_argument_errors(pkg):
    print("[case] domain argument errors", flush=True)
    torch.manual_seed(3)
    ix = pkg.Index(32, 1000, pkg.STORE_BF16, 8, 16, DEV)
    L = pkg.load_library()
    q = torch.zeros((4, 32), device=DEV)
    o_s = torch.empty((4, 4), device=DEV)
    o_i = torch.empty((4, 4), dtype=torch.int64, device=DEV)
    assert L.ic_search_domains(ix.handle, q.data_ptr(), 4, 4, 0.0, None, None, o_s.data_ptr(), o_i.data_ptr()) == 1
    assert L.ic_index_set_domains(ix.handle, None, None, 3) == 1
    assert L.ic_index_set_domains(ix.handle, None, None, 0) == 0
    # ids out of range are skipped
    ix.append(torch.randn(10, 32, device=DEV), None)
    ix.set_domains(torch.tensor([-1, 3, 10, 999], device=DEV), torch.tensor([5, 5, 5, 5], dtype=torch.int32, device=DEV))
    s, i = ix.search_domains(torch.randn(2, 32, device=DEV), 10, torch.tensor([0, 5], dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    got = i.cpu().numpy()
    assert 3 not in got[0].tolist() and 3 in got[1].tolist()
    assert sorted(got[0].tolist()) == [-1, 0, 1, 2, 4, 5, 6, 7, 8, 9] and got[0, -1] == -1   # 9 rows visible to domain 0
    assert sorted(got[1].tolist()) == list(range(10))
    ix.close()
