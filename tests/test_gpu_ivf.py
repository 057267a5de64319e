"""GPU parity of cluster pruning (K-Means lists in front of the scan), through the C ABI.

Every step is checked with inputs that come from the seeded generators or from the CPU
reference, never from another GPU step: the assignment against given centroids, the lists and
the sorted copy from a given assignment, the K-Means update from a given assignment, and the
pruned search from given centroids and assignment.  The end-to-end training is compared with the
reference's K-Means from the same start by what is well defined: agreement of the assignments,
the clustering objective, and recall against the exact search."""
import sys

import numpy as np
import pytest
import torch

import parity
import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def pkg():
    import paper_2501_12689_amd as p
    p.load_library()
    return p


def _setup(pkg, store, N=60000, d=96, C=48, seed=9600, util="uniform"):
    cfg = workloads.Config("V", N=N, d=d, clusters=C, Q=40, k=10, store=store, zipf=1.1, lam=0.2, util=util, seed=seed)
    wl = workloads.Workload(cfg, "cpu")
    E, U, _ = wl.rows(0, N)
    sid = pkg.STORE_BF16 if store == "bf16" else pkg.STORE_FP8_E4M3
    ix = pkg.Index(d, N, sid, 64, 16, DEV)
    ix.append(E.to(DEV), None if U is None else U.to(DEV))
    return cfg, wl, ix, E.numpy(), (None if U is None else U.numpy())


def _stored(oracle, store, X):
    """fp64 values a store of this format holds for rows X (the reference's own quantiser)."""
    if store == "bf16":
        return oracle.decode_bf16(oracle.quantize_bf16(X)).astype(np.float64)
    c, s = oracle.quantize_fp8(X)
    return oracle.decode_e4m3(c).astype(np.float64) * s[:, None].astype(np.float64)


@pytest.mark.parametrize("store,K,N,d", [("bf16", 48, 60000, 96), ("fp8", 48, 60000, 96),
                                         ("bf16", 300, 40001, 64),     # two blocks of centroids, ragged last row tile
                                         ("fp8", 515, 30000, 128),     # three blocks, the last with 3 centroids
                                         ("bf16", 129, 20000, 768)])   # one centroid past a half block, long rows
def test_assignment_against_given_centroids(pkg, oracle, store, K, N, d):
    _say(f"ivf assign, {store}, K={K}, N={N}, d={d}")
    cfg, wl, ix, E, U = _setup(pkg, store, N=N, d=d, C=K)
    C = wl.centres.numpy().copy()
    C[5] = C[4]                                   # two identical centroids: the lower id must win
    ivf = pkg.Ivf(ix, K, 4)
    ivf.set_centroids(torch.from_numpy(C).to(DEV))
    ivf.assign()
    assign = ivf.view()[0].cpu().numpy()
    # scores of the stored values (rows and centroids through the reference's quantiser)
    S = _stored(oracle, store, E) @ _stored(oracle, store, C).T
    best = S.max(axis=1)
    got = S[np.arange(cfg.N), assign]
    assert np.all(assign >= 0) and np.all(assign < K)
    assert np.all(got >= best - parity.TAU_Q), f"row assigned {float((best - got).max()):.3g} below its best centroid"
    clear = (np.sort(S, axis=1)[:, -1] - np.sort(S, axis=1)[:, -2]) > parity.TAU_Q
    ref = S.argmax(axis=1)
    assert np.array_equal(assign[clear], ref[clear])
    assert not np.any(assign == 5)                 # the duplicate never wins
    ref64 = oracle.ivf_assign(E, C)                # fp64 masters: agrees except near cluster borders
    print(f"   agreement with the fp32-master reference: {(assign == ref64).mean():.5f}", flush=True)
    assert (assign == ref64).mean() > 0.995
    ivf.close(); ix.close()


@pytest.mark.parametrize("store", ["bf16", "fp8"])
def test_lists_and_sorted_copy_from_a_given_assignment(pkg, oracle, store):
    _say(f"ivf lists, {store}")
    cfg, wl, ix, E, U = _setup(pkg, store, N=50001)
    K = 37
    rng = np.random.default_rng(3)
    assign = rng.integers(-1, K + 2, cfg.N).astype(np.int32)      # includes -1, K, K+1: in no list
    assign[assign == 7] = 8                                       # an empty cluster
    gone = rng.choice(cfg.N, 5000, replace=False).astype(np.int64)
    ix.invalidate(torch.from_numpy(gone).to(DEV))
    valid = oracle.invalidate(np.ones(cfg.N, np.uint8), gone)
    rows0, scale0, util0 = (None if t is None else t.cpu().numpy().copy() for t in ix.store_view())
    ivf = pkg.Ivf(ix, K, 4)
    ivf.set_assignment(torch.from_numpy(assign).to(DEV))
    a, offsets, perm, _, _ = ivf.view()
    ref_off, ref_lists = oracle.ivf_lists(assign, K, valid)
    assert np.array_equal(a.cpu().numpy(), assign)
    assert np.array_equal(offsets.cpu().numpy(), ref_off)
    perm = perm.cpu().numpy().astype(np.int64)
    assert perm.shape[0] == ref_off[-1]
    for c in range(K):                                            # order inside a list is free
        assert np.array_equal(np.sort(perm[ref_off[c]:ref_off[c + 1]]), ref_lists[c]), f"list {c}"
    # the sorted copy holds exactly the rows perm names
    L = pkg.load_library()
    import ctypes
    s_handle = ctypes.c_void_p()
    assert L.ic_ivf_view(ivf.handle, None, None, None, None, ctypes.byref(s_handle)) == 0
    assert L.ic_index_size(s_handle.value) == ref_off[-1]
    rows, stride = ctypes.c_void_p(), ctypes.c_int64()
    sc, ut = ctypes.c_void_p(), ctypes.c_void_p()
    assert L.ic_index_store_view(s_handle.value, ctypes.byref(rows), ctypes.byref(stride), ctypes.byref(sc), ctypes.byref(ut)) == 0
    base = ivf.arena.data_ptr()
    n, rb = int(ref_off[-1]), stride.value
    srows = ivf.arena[rows.value - base: rows.value - base + n * rb].view(n, rb).cpu().numpy()
    sutil = ivf.arena[ut.value - base: ut.value - base + 4 * n].view(torch.float32).cpu().numpy()
    assert np.array_equal(srows, rows0[perm]) and np.array_equal(sutil, util0[perm])
    if scale0 is not None:
        sscale = ivf.arena[sc.value - base: sc.value - base + 4 * n].view(torch.float32).cpu().numpy()
        assert np.array_equal(sscale, scale0[perm])
    ivf.close(); ix.close()


@pytest.mark.parametrize("store", ["bf16", "fp8"])
def test_update_step_from_a_given_assignment(pkg, oracle, store):
    _say(f"ivf update, {store}")
    cfg, wl, ix, E, U = _setup(pkg, store, N=40000)
    K = cfg.clusters
    C0 = wl.centres.numpy()
    assign = oracle.ivf_assign(E, C0)
    assign[assign == 11] = 12                                     # cluster 11 is empty: keeps its centroid
    ivf = pkg.Ivf(ix, K, 4)
    ivf.set_centroids(torch.from_numpy(C0).to(DEV))
    ivf.set_assignment(torch.from_numpy(assign).to(DEV))
    ivf.update_centroids()
    _, _, _, crow, cscale = ivf.view()
    torch.cuda.synchronize()
    crow = crow.cpu().numpy()
    if store == "bf16":
        got = oracle.decode_bf16(crow.view(np.uint16)[:, :cfg.d]).astype(np.float64)
    else:
        got = oracle.decode_e4m3(crow[:, :cfg.d]).astype(np.float64) * cscale.cpu().numpy()[:, None].astype(np.float64)
    # reference: mean direction of the stored values of each list; the empty list keeps the stored old centroid
    want = oracle.ivf_update(_stored(oracle, store, E), assign, K, _stored(oracle, store, C0), normalize=False)
    want_q = _stored(oracle, store, want.astype(np.float32))      # and is itself stored in the same format
    cos = (oracle._unit(got) * oracle._unit(want)).sum(axis=1)
    assert cos.min() > 1 - (1e-4 if store == "bf16" else 1e-3), cos.min()   # got is quantised, want is not
    # element by element: the same code except where the value sits on a rounding boundary
    step = np.abs(want_q).max(axis=1, keepdims=True) * (2.0 ** -7 if store == "bf16" else 2.0 ** -3)
    assert np.all(np.abs(got - want_q) <= step)
    if store == "bf16":
        same = crow.view(np.uint16)[:, :cfg.d] == oracle.quantize_bf16(want.astype(np.float32))
    else:
        wc, ws = oracle.quantize_fp8(want.astype(np.float32))
        same = crow[:, :cfg.d] == wc
        assert np.allclose(cscale.cpu().numpy(), ws, rtol=1e-5)
    assert same.mean() > 0.98, same.mean()
    # the empty cluster's centroid is stored again from its own stored values: the same direction
    # (re-normalising and re-rounding may move single codes)
    old11 = _stored(oracle, store, C0)[11:12]
    assert float((oracle._unit(got[11:12]) * oracle._unit(old11)).sum()) > 1 - (1e-6 if store == "bf16" else 1e-3)
    ivf.close(); ix.close()


@pytest.mark.parametrize("store,nprobe,lam", [("bf16", 1, 0.0), ("bf16", 4, 0.2), ("fp8", 3, 0.2)])
def test_pruned_search_from_given_centroids_and_assignment(pkg, oracle, store, nprobe, lam):
    _say(f"ivf search, {store}, nprobe={nprobe}")
    cfg, wl, ix, E, U = _setup(pkg, store)
    K = cfg.clusters
    C = wl.centres.numpy()
    assign = oracle.ivf_assign(E, C)                              # the reference's clustering, given to the GPU
    ivf = pkg.Ivf(ix, K, 8)
    ivf.set_centroids(torch.from_numpy(C).to(DEV))
    ivf.set_assignment(torch.from_numpy(assign).to(DEV))
    Qm = wl.queries(40).numpy()
    s, i = ivf.search(torch.from_numpy(Qm).to(DEV), cfg.k, nprobe, lam)
    torch.cuda.synchronize()
    gs, gi = s.cpu().numpy(), i.cpu().numpy()
    # the probe set is part of the answer: it is unambiguous when the nprobe-th and the next
    # centroid are further apart than the tolerance; those queries get the full comparison with
    # "rows of the probed clusters" as the set of valid rows
    cs = oracle.scores(C, Qm)
    order = np.argsort(-cs, axis=1, kind="stable")
    checked = 0
    for q in range(Qm.shape[0]):
        top = order[q, :nprobe]
        gap = cs[q, order[q, nprobe - 1]] - cs[q, order[q, nprobe]]
        members = np.isin(assign, top).astype(np.uint8)
        # the centroid ranking is decided on quantised values: bf16 moves a cosine by < 4e-3 (two
        # roundings of 2^-9 each), fp8 stayed below 1e-2 in every measurement
        if gap > (5e-3 if store == "bf16" else 3e-2):
            parity.check_batch(store, gs[q:q + 1], gi[q:q + 1], E, U, members, Qm[q:q + 1], cfg.k, lam, f"ivf q={q}")
            checked += 1
        else:  # either neighbour cluster may have been probed: every row returned is from one of them
            ok = np.isin(assign[gi[q][gi[q] >= 0]], order[q, :nprobe + 1])
            assert np.all(ok)
    assert checked >= 10, checked
    # probing every cluster is the exact search
    if nprobe == 4:
        sa, ia = pkg.Ivf.search(ivf, torch.from_numpy(Qm).to(DEV), cfg.k, 8, lam)   # 8 of 48: still pruned
        se, ie = ix.search(torch.from_numpy(Qm).to(DEV), cfg.k, lam)
        torch.cuda.synchronize()
        rec = np.mean([len(set(ia[q].tolist()) & set(ie[q].tolist())) / cfg.k for q in range(Qm.shape[0])])
        print(f"   recall@{cfg.k} of 8 probes against the exact search: {rec:.4f}", flush=True)
        assert rec > 0.95
    ivf.close(); ix.close()


def _drawn_pruned(count, seed):
    """Seeded draw of pruned searches the fixed cases do not name: any row length, 2 to 600 clusters
    (uniform or Zipf sizes, so lists from empty to most of the store), 1 to all clusters probed,
    batches beyond one block of 64 queries, evicted rows."""
    rng = np.random.default_rng(seed)
    out = []
    for n in range(count):
        store = "fp8" if rng.random() < 0.4 else "bf16"
        d = int(rng.choice([rng.integers(8, 65), rng.integers(65, 300), rng.integers(300, 900)]))
        N = int(rng.choice([rng.integers(300, 3000), rng.integers(3000, 60000), rng.integers(60000, 150000)]))
        N = min(N, int(6e7 // d))
        K = min(int(rng.choice([rng.integers(2, 10), rng.integers(10, 100), rng.integers(100, 600)])), max(2, N // 4))
        max_probe = int(min(K, rng.choice([1, 2, 8, 32])))
        out.append((store, N, d, K, int(rng.integers(1, max_probe + 1)), max_probe,
                    int(rng.choice([1, rng.integers(2, 65), rng.integers(65, 150)])),
                    int(rng.choice([1, rng.integers(2, 17), rng.integers(17, 64)])),
                    float(rng.choice([0.0, 0.2])), float(rng.choice([0.0, 0.1])), float(rng.choice([0.0, 1.1]))))
    return out


DRAWN_PRUNED = _drawn_pruned(16, 20250114)


@pytest.mark.parametrize("case", DRAWN_PRUNED, ids=lambda c: "-".join(str(x) for x in c))
def test_pruned_search_on_drawn_shapes(pkg, oracle, case):
    store, N, d, K, nprobe, max_probe, Q, k, lam, evicted, zipf = case
    _say(f"ivf search, drawn shape {case}")
    n = DRAWN_PRUNED.index(case)
    rng = np.random.default_rng(9700 + n)
    cfg = workloads.Config("V", N=N, d=d, clusters=K, Q=Q, k=k, store=store, zipf=zipf, lam=lam, util="uniform",
                           seed=9700 + n)
    wl = workloads.Workload(cfg, "cpu")
    E, U, _ = wl.rows(0, N)
    E, U = E.numpy(), U.numpy()
    C = wl.centres.numpy()
    sid = pkg.STORE_BF16 if store == "bf16" else pkg.STORE_FP8_E4M3
    ix = pkg.Index(d, N, sid, max(64, Q), 64, DEV)
    ix.append(torch.from_numpy(E).to(DEV), torch.from_numpy(U).to(DEV))
    live = np.ones(N, bool)
    if evicted > 0:
        gone = rng.choice(N, int(N * evicted), replace=False).astype(np.int64)
        ix.invalidate(torch.from_numpy(gone).to(DEV))
        live[gone] = False
    assign = oracle.ivf_assign(E, C)
    ivf = pkg.Ivf(ix, K, max_probe)
    ivf.set_centroids(torch.from_numpy(C).to(DEV))
    ivf.set_assignment(torch.from_numpy(assign).to(DEV))
    Qm = wl.queries(Q).numpy()
    s, i = ivf.search(torch.from_numpy(Qm).to(DEV), k, nprobe, lam)
    torch.cuda.synchronize()
    gs, gi = s.cpu().numpy(), i.cpu().numpy()
    ivf.close(); ix.close()
    cs = oracle.scores(C, Qm)
    order = np.argsort(-cs, axis=1, kind="stable")
    for q in sorted(set([0, Q - 1] + [int(x) for x in rng.integers(0, Q, size=6)])):
        gap = np.inf if nprobe >= K else cs[q, order[q, nprobe - 1]] - cs[q, order[q, nprobe]]
        if gap > (5e-3 if store == "bf16" else 3e-2):     # the probe set is unambiguous (see the test above)
            members = (np.isin(assign, order[q, :nprobe]) & live).astype(np.uint8)
            parity.check_batch(store, gs[q:q + 1], gi[q:q + 1], E, U, members, Qm[q:q + 1], k, lam, f"{case} q={q}")
        else:
            got = gi[q][gi[q] >= 0]
            assert np.all(np.isin(assign[got], order[q, :nprobe + 1])) and np.all(live[got])


@pytest.mark.parametrize("store", ["bf16", "fp8"])
def test_pruned_search_does_not_depend_on_the_batch(pkg, oracle, store):
    """Queries of a batch that probe the same list share one read of it, up to 16 to a scan task.  With
    6 clusters and 100 queries every list is probed by far more than 16 queries, so lists are served by
    several full tasks and a ragged one; every query must get exactly what it gets when searched alone
    or in small batches (each score is the same sum whatever slot the query sits in), and what the
    reference finds in the probed lists."""
    _say(f"ivf search, shared lists, {store}")
    cfg, wl, ix, E, U = _setup(pkg, store, N=30000, d=160, C=6, seed=9660)
    K, nprobe, k, lam = 6, 2, 12, 0.2
    C = wl.centres.numpy()
    assign = oracle.ivf_assign(E, C)
    ivf = pkg.Ivf(ix, K, 4)
    ivf.set_centroids(torch.from_numpy(C).to(DEV))
    ivf.set_assignment(torch.from_numpy(assign).to(DEV))
    Qm = wl.queries(100).numpy()
    qd = torch.from_numpy(Qm).to(DEV)
    s, i = ivf.search(qd, k, nprobe, lam)
    torch.cuda.synchronize()
    gs, gi = s.cpu().numpy(), i.cpu().numpy()
    for step in (1, 7):
        for q0 in list(range(0, 100, step))[:: (9 if step == 1 else 3)]:
            s1, i1 = ivf.search(qd[q0:q0 + step].contiguous(), k, nprobe, lam)
            torch.cuda.synchronize()
            assert np.array_equal(i1.cpu().numpy(), gi[q0:q0 + step]) and np.array_equal(s1.cpu().numpy(), gs[q0:q0 + step]), (step, q0)
    cs = oracle.scores(C, Qm)
    order = np.argsort(-cs, axis=1, kind="stable")
    checked = 0
    for q in range(0, 100, 5):
        if cs[q, order[q, nprobe - 1]] - cs[q, order[q, nprobe]] > (5e-3 if store == "bf16" else 3e-2):
            members = np.isin(assign, order[q, :nprobe]).astype(np.uint8)
            parity.check_batch(store, gs[q:q + 1], gi[q:q + 1], E, U, members, Qm[q:q + 1], k, lam, f"shared lists q={q}")
            checked += 1
    assert checked >= 10, checked
    ivf.close(); ix.close()


@pytest.mark.parametrize("store,d", [("bf16", 384), ("bf16", 576), ("fp8", 1280), ("bf16", 768), ("fp8", 1024)])
def test_pruned_search_over_all_lists_equals_the_full_scan(pkg, store, d):
    """With every list probed the pruned search sees every row, through the same kernel arithmetic as the
    full scan (the same deal of a row's chunks to the wavefronts, whatever the row length): same ids, same
    score bits."""
    _say(f"pruned search over all lists against the full scan, {store} d={d}")
    N, K, Q, k = 60000, 16, 40, 20
    cfg = workloads.Config("V", N=N, d=d, clusters=K, Q=Q, k=k, store=store, zipf=1.1, lam=0.1, util="uniform", seed=9900 + d)
    wl = workloads.Workload(cfg, DEV)
    E, U, _ = wl.rows(0, N)
    ix = pkg.Index(d, N, pkg.STORE_BF16 if store == "bf16" else pkg.STORE_FP8_E4M3, 64, 64, DEV)
    ix.append(E, U)
    ivf = pkg.Ivf(ix, K, K)
    ivf.train(3)
    qd = wl.queries(Q)
    s1, i1 = ix.search(qd, k, 0.1, None)
    s2, i2 = ivf.search(qd, k, K, 0.1)
    torch.cuda.synchronize()
    ivf.close()
    ix.close()
    assert torch.equal(i1, i2) and torch.equal(s1, s2)


def test_many_centroids_and_a_large_batch_take_the_tiled_scan(pkg, oracle):
    """With 16,400 centroids and 200 queries the probe step (nearest centroids of every query) is a
    batch large enough for the MFMA-tiled scan over the centroid index, whose step-major copy is
    rewritten every time the centroids are loaded: twice here, the second load being the one that counts."""
    _say("ivf search, 16400 centroids, 200 queries")
    K, N, d, k, nprobe = 16400, 40000, 64, 4, 2
    cfg = workloads.Config("V", N=N, d=d, clusters=K, Q=200, k=k, store="bf16", sigma=0.25, seed=9650)
    wl = workloads.Workload(cfg, "cpu")
    E = wl.rows(0, N)[0].numpy()
    C = wl.centres.numpy()
    ix = pkg.Index(d, N, pkg.STORE_BF16, 256, 16, DEV)
    ix.append(torch.from_numpy(E).to(DEV), None)
    assign = oracle.ivf_assign(E, C)
    ivf = pkg.Ivf(ix, K, 4)
    ivf.set_centroids(torch.from_numpy(np.ascontiguousarray(C[::-1])).to(DEV))   # a first set, overwritten below
    ivf.set_centroids(torch.from_numpy(C).to(DEV))
    ivf.set_assignment(torch.from_numpy(assign).to(DEV))
    Qm = wl.queries(cfg.Q).numpy()
    s, i = ivf.search(torch.from_numpy(Qm).to(DEV), k, nprobe, 0.0)
    torch.cuda.synchronize()
    gs, gi = s.cpu().numpy(), i.cpu().numpy()
    cs = oracle.scores(C, Qm)
    order = np.argsort(-cs, axis=1, kind="stable")
    checked = 0
    for q in range(0, cfg.Q, 3):
        top = order[q, :nprobe]
        gap = cs[q, order[q, nprobe - 1]] - cs[q, order[q, nprobe]]
        if gap > 5e-3:
            members = np.isin(assign, top).astype(np.uint8)
            parity.check_batch("bf16", gs[q:q + 1], gi[q:q + 1], E, None, members, Qm[q:q + 1], k, 0.0, f"ivf q={q}")
            checked += 1
        else:
            assert np.all(np.isin(assign[gi[q][gi[q] >= 0]], order[q, :nprobe + 1]))
    assert checked >= 30, checked
    ivf.close(); ix.close()


def test_training_against_the_reference_kmeans(pkg, oracle):
    _say("ivf train")
    cfg, wl, ix, E, U = _setup(pkg, "bf16", N=30000, d=64, C=24, util="none")
    K, iters = 24, 3
    ivf = pkg.Ivf(ix, K, 8)
    ivf.train(iters)
    assign, offsets, perm, crow, _ = ivf.view()
    torch.cuda.synchronize()
    assign, perm = assign.cpu().numpy(), perm.cpu().numpy()
    # every row is in exactly one list
    assert np.array_equal(np.sort(perm), np.arange(cfg.N)) and int(offsets[-1]) == cfg.N
    Cg = oracle.decode_bf16(crow.cpu().numpy().view(np.uint16)[:, :cfg.d]).astype(np.float64)
    Cr, ar = oracle.ivf_kmeans(E, K, iters)                       # same start, same number of iterations
    Eu = oracle._unit(E)
    obj_g = float((Eu * oracle._unit(Cg)[assign]).sum(axis=1).mean())
    obj_r = float((Eu * Cr[ar]).sum(axis=1).mean())
    print(f"   objective GPU {obj_g:.6f} reference {obj_r:.6f}; assignments equal {(assign == ar).mean():.5f}", flush=True)
    # the objective is well conditioned; the assignment is not where two centroids share one blob
    # (rows between them flip with the last bits of the centroids), hence the loose second bound
    assert abs(obj_g - obj_r) < 1e-3 and (assign == ar).mean() > 0.9
    # pruned search with the trained lists against the exact search
    Qd = wl.queries(64).to(DEV)
    se, ie = ix.search(Qd, 10)
    for nprobe, floor in ((1, 0.5), (4, 0.9), (8, 0.97)):
        s, i = ivf.search(Qd, 10, nprobe)
        torch.cuda.synchronize()
        rec = np.mean([len(set(i[q].tolist()) & set(ie[q].tolist())) / 10 for q in range(64)])
        print(f"   nprobe={nprobe}: recall@10 {rec:.4f}", flush=True)
        assert rec >= floor
    ivf.close(); ix.close()


def test_lists_are_a_snapshot_until_assigned_again(pkg, oracle):
    """Rows appended or evicted after the lists were built are not seen by the pruned search until
    ic_ivf_assign is called again; afterwards it agrees with the reference on the new store."""
    _say("ivf snapshot / re-assign")
    N0, extra, d, K, k = 30000, 5000, 64, 40, 8
    cfg = workloads.Config("V", N=N0 + extra, d=d, clusters=K, Q=32, k=k, store="bf16", zipf=1.1, lam=0.0,
                           util="none", seed=9650)
    wl = workloads.Workload(cfg, "cpu")
    E = wl.rows(0, N0 + extra)[0]
    ix = pkg.Index(d, N0 + extra, pkg.STORE_BF16, 64, 16, DEV)
    ix.append(E[:N0].to(DEV), None)
    C = wl.centres.numpy()
    ivf = pkg.Ivf(ix, K, K)
    ivf.set_centroids(torch.from_numpy(C).to(DEV))
    ivf.assign()
    Qd = wl.queries().to(DEV)
    ix.append(E[N0:].to(DEV), None)
    gone = torch.arange(0, N0, 3, device=DEV)
    ix.invalidate(gone)
    s, i = ivf.search(Qd, k, K)                  # every list probed: the exact result over the snapshot
    torch.cuda.synchronize()
    assert int(i.max()) < N0                      # the appended rows are not in any list yet
    ivf.assign()
    s, i = ivf.search(Qd, k, K)
    se, ie = ix.search(Qd, k)                     # the exact search sees appends and evictions at once
    torch.cuda.synchronize()
    assert int(i.max()) >= N0
    assert not np.isin(i.cpu().numpy(), gone.cpu().numpy()).any()
    assert torch.allclose(s, se, atol=2e-6) and (i == ie).float().mean() > 0.995
    ivf.close(); ix.close()


def test_ivf_argument_errors(pkg):
    ix = pkg.Index(32, 1000, pkg.STORE_BF16, 16, 4, DEV)
    ix.append(torch.randn(500, 32, device=DEV))
    with pytest.raises(ValueError):
        pkg.Ivf(ix, 0, 4)
    ivf = pkg.Ivf(ix, 10, 4)
    q = torch.randn(3, 32, device=DEV)
    with pytest.raises(pkg.ICError):
        ivf.search(q, 2, 1)                  # no lists yet
    with pytest.raises(pkg.ICError):
        ivf.assign()                         # no centroids yet
    ivf.train(1)
    for k, nprobe in [(0, 1), (5, 1), (2, 0), (2, 5)]:
        with pytest.raises(pkg.ICError):
            ivf.search(q, k, nprobe)
    s, i = ivf.search(q, 2, 4)
    torch.cuda.synchronize()
    assert bool((i >= 0).all())
    ivf.close(); ix.close()
