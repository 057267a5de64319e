"""The entry point that allocates nothing (``ic_search_static``: the search scratch lies in a static
device array inside the library) against ``ic_search`` on the same index, through the C ABI.

Both run the same kernels on the same prepared queries and the result does not depend on the
launch shape, so the two must agree bit for bit; ``ic_search`` itself is checked against the CPU
reference here as well.  Two calls in a row share the static array: the second one is smaller (fewer
queries, smaller k, a smaller index) and must not see anything the first one left behind.
"""
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
    assert torch.cuda.is_available(), "these tests need the GPU"
    return p


def _index(pkg, cfg, max_k):
    wl = workloads.Workload(cfg, "cpu")
    E, U, M = wl.rows(0, cfg.N)
    sid = pkg.STORE_BF16 if cfg.store == "bf16" else pkg.STORE_FP8_E4M3
    ix = pkg.Index(cfg.d, cfg.N, sid, 64, max_k, DEV)
    ix.append(E.to(DEV), None if U is None else U.to(DEV))
    return ix, wl, E, U, M


def _both(pkg, ix, Qm, k, lam, M):
    qd = Qm.to(DEV)
    md = None if M is None else M.to(DEV)
    s0, i0 = ix.search(qd, k, lam, md)
    s1 = torch.full((Qm.shape[0], k), 7.0, dtype=torch.float32, device=DEV)
    i1 = torch.full((Qm.shape[0], k), -7, dtype=torch.int64, device=DEV)
    pkg.ic_search_static(ix.handle, qd, k, lam, md, s1, i1)
    torch.cuda.synchronize()
    return s0.cpu().numpy(), i0.cpu().numpy(), s1.cpu().numpy(), i1.cpu().numpy()


@pytest.mark.parametrize("store", ["bf16", "fp8"])
def test_static_scratch_search_equals_ic_search_twice_in_a_row(pkg, store):
    _say(f"ic_search_static vs ic_search, {store}: large call then small call")
    big = workloads.Config("S1", N=300_000, d=768, clusters=64, Q=64, k=64, store=store, zipf=1.1, lam=0.3,
                           util="uniform", p_valid=0.9, seed=9100)
    small = workloads.Config("S2", N=20_000, d=200, clusters=16, Q=7, k=10, store=store, seed=9101)
    ixb, wlb, Eb, Ub, Mb = _index(pkg, big, 128)
    ixs, wls, Es, Us, Ms = _index(pkg, small, 16)
    calls = [(ixb, wlb.queries(64), 100, big.lam, Mb, Eb, Ub),      # pilot, 64 queries, k = 100
             (ixs, wls.queries(7), 10, 0.0, None, Es, None),         # no bias, no pilot, another index
             (ixb, wlb.queries(3, batch=1), 5, big.lam, Mb, Eb, Ub)]  # the first index again, 3 queries
    for n, (ix, Qm, k, lam, M, E, U) in enumerate(calls):
        s0, i0, s1, i1 = _both(pkg, ix, Qm, k, lam, M)
        assert np.array_equal(i0, i1), f"call {n}: ids differ"
        assert np.array_equal(s0, s1), f"call {n}: scores differ"
        parity.check_batch(store, s1, i1, E.numpy(), None if U is None else U.numpy(),
                           None if M is None else M.numpy(), Qm.numpy(), k, lam, f"static call {n}",
                           queries=range(0, Qm.shape[0], 9))
    ixb.close(); ixs.close()


def test_static_scratch_search_limits_and_edges(pkg):
    _say("ic_search_static: limits, empty index, k > rows")
    L = pkg.load_library()
    cfg = workloads.Config("S3", N=3000, d=96, clusters=4, Q=8, k=8, seed=9102)
    ix, wl, E, U, M = _index(pkg, cfg, 128)
    qd = wl.queries(65).to(DEV)
    s = torch.empty(65, 8, dtype=torch.float32, device=DEV)
    i = torch.empty(65, 8, dtype=torch.int64, device=DEV)
    with pytest.raises(pkg.ICError) as err:                       # more queries than the scratch is laid out for
        pkg.ic_search_static(ix.handle, qd, 8, 0.0, None, s, i)
    assert err.value.status == 5
    with pytest.raises(pkg.ICError) as err:                       # k beyond the index's max_k
        pkg.ic_search_static(ix.handle, qd[:4].contiguous(), 129, 0.0, None, s, i)
    assert err.value.status == 1
    assert L.ic_search_static(None, qd.data_ptr(), 4, 8, 0.0, None, s.data_ptr(), i.data_ptr()) == 1
    # k larger than the number of valid rows: padded tail, as ic_search
    mask = torch.zeros(cfg.N, dtype=torch.uint8)
    mask[[5, 77, 2999]] = 1
    s0, i0, s1, i1 = _both(pkg, ix, wl.queries(4), 8, 0.0, mask)
    assert np.array_equal(i0, i1) and np.array_equal(s0, s1)
    assert np.all(i1[:, 3:] == -1) and np.all(np.isneginf(s1[:, 3:]))
    assert all(set(r[:3].tolist()) == {5, 77, 2999} for r in i1)
    ix.close()
    # empty index: every entry is padding
    ixe = pkg.Index(96, 100, pkg.STORE_BF16, 64, 16, DEV)
    s1 = torch.zeros(4, 8, dtype=torch.float32, device=DEV)
    i1 = torch.zeros(4, 8, dtype=torch.int64, device=DEV)
    pkg.ic_search_static(ixe.handle, wl.queries(4).to(DEV), 8, 0.0, None, s1, i1)
    torch.cuda.synchronize()
    assert bool((i1 == -1).all()) and bool(torch.isneginf(s1).all())
    ixe.close()
    # an index larger than the scratch's bias array is refused
    rows = 4_194_304 + 1
    big = pkg.Index(1, rows, pkg.STORE_FP8_E4M3, 64, 16, DEV)
    big.append(torch.ones(rows, 1, dtype=torch.float32, device=DEV))
    with pytest.raises(pkg.ICError) as err:
        pkg.ic_search_static(big.handle, torch.ones(1, 1, device=DEV), 8, 0.0, None, s1, i1)
    assert err.value.status == 5
    big.close()
