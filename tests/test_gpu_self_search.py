"""GPU parity of self-search (stored rows as queries, each left out of its own result), through
the C ABI."""
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


CASES = [
    # store, N, d, first_row, count, k, lam, util, p_valid, max_queries
    ("bf16", 40000, 96, 100, 50, 5, 0.0, "none", 1.0, 64),
    ("fp8", 30000, 128, 29990, 10, 1, 0.2, "uniform", 0.9, 16),        # the last rows of the store
    ("bf16", 280000, 128, 1000, 300, 3, 0.1, "beta25", 0.95, 512),     # tiled scan, one chunk
    ("fp8", 270000, 64, 0, 300, 1, 0.0, "none", 1.0, 128),            # tiled scan, chunks of 128 + a streamed rest
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "-".join(str(x) for x in c))
def test_self_search(pkg, oracle, case):
    store, N, d, first, count, k, lam, util, pv, max_q = case
    print(f"[case] self-search {case}", flush=True)
    sys.stdout.flush()
    cfg = workloads.Config("S", N=N, d=d, clusters=32, Q=8, k=k, store=store, zipf=1.1, lam=lam, util=util,
                           p_valid=pv, seed=9500 + CASES.index(case))
    wl = workloads.Workload(cfg, "cpu")
    E, U, M = wl.rows(0, N)
    E[first + 3] = E[first + 1]                      # a duplicate pair inside the queried range
    sid = pkg.STORE_BF16 if store == "bf16" else pkg.STORE_FP8_E4M3
    ix = pkg.Index(d, N, sid, max_q, k + 1, DEV)
    ix.append(E.to(DEV), None if U is None else U.to(DEV))
    md = None if M is None else M.to(DEV)
    s, i = ix.self_search(first, count, k, lam, md)
    torch.cuda.synchronize()
    gs, gi = s.cpu().numpy(), i.cpu().numpy()
    En, Un = E.numpy(), (None if U is None else U.numpy())
    Mn = np.ones(N, np.uint8) if M is None else M.numpy()
    rows = np.arange(first, first + count)
    assert not np.any(gi == rows[:, None]), "a row returned itself"
    if Mn[first + 1] and Mn[first + 3] and lam == 0.0:
        assert gi[1, 0] == first + 3 and gi[3, 0] == first + 1 and abs(gs[1, 0] - 1.0) < parity.TAU[store]
    # every sampled row: the ordinary checks with that row masked out in addition
    for j in sorted(set(list(range(0, count, max(1, count // 10))) + [1, 3, count - 1])):
        Mr = Mn.copy()
        Mr[rows[j]] = 0
        parity.check_batch(store, gs[j:j + 1], gi[j:j + 1], En, Un, Mr, En[rows[j]:rows[j] + 1], k, lam,
                           f"self-search row {rows[j]}")
    # the same rows given as ordinary fp32 queries: the query preparation reproduces the stored row
    # bit for bit, so the scores are those of the self-search with the row itself in front
    nq = min(count, max_q)
    s2, i2 = ix.search(E[first:first + nq].contiguous().to(DEV), k + 1, lam, md)
    torch.cuda.synchronize()
    s2, i2 = s2.cpu().numpy(), i2.cpu().numpy()
    same = 0
    for j in range(nq):
        keep = [p for p in range(k + 1) if i2[j, p] != rows[j]][:k]
        # the two calls may be served by different kernels (a tile full of self-matches overflows the
        # ordinary search's hit list and is redone by the streaming scan): scores agree to rounding
        assert np.allclose(s2[j, keep], gs[j], atol=2e-6), f"row {rows[j]}"
        same += int(np.array_equal(i2[j, keep], gi[j]))
    assert same >= 0.99 * nq
    ix.close()


def test_self_search_argument_errors(pkg):
    ix = pkg.Index(32, 1000, pkg.STORE_BF16, 16, 4, DEV)
    ix.append(torch.randn(500, 32, device=DEV))
    for first, count, k in [(-1, 10, 1), (495, 10, 1), (0, 10, 4), (0, 10, 0)]:
        with pytest.raises(pkg.ICError):
            ix.self_search(first, count, k)
    s, i = ix.self_search(10, 0, 2)
    assert s.shape == (0, 2)
    ix.close()
