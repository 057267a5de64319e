"""A search is a fixed sequence of kernel launches on the index's stream (no allocation, no host
synchronisation, no memset nodes), so a caller can capture it into a HIP graph and replay it:
what launch-bound small caches need.  Every replay is checked against the eager call on the same
inputs, with eager work and synchronisations between the replays."""
import sys

import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def pkg():
    import paper_2501_12689_amd as p
    p.load_library()
    return p


@pytest.mark.parametrize("case", [("bf16", 100000, 384, 64, 10, 0.0), ("fp8", 40000, 256, 16, 32, 0.2),
                                  ("bf16", 300000, 128, 300, 16, 0.1)],
                         ids=lambda c: "-".join(str(x) for x in c))
def test_search_replayed_from_a_graph_equals_eager(pkg, case):
    store, N, d, Q, k, lam = case
    print(f"[case] graph replay {case}", flush=True)
    sys.stdout.flush()
    cfg = workloads.Config("H", N=N, d=d, clusters=32, Q=Q, k=k, store=store, zipf=1.1, lam=lam,
                           util="uniform" if lam else "none", p_valid=0.9, seed=9900)
    wl = workloads.Workload(cfg, DEV)
    E, U, M = wl.rows(0, N)
    sid = pkg.STORE_BF16 if store == "bf16" else pkg.STORE_FP8_E4M3
    ix = pkg.Index(d, N, sid, Q, k, DEV)
    ix.append(E, U)
    batches = [wl.queries(Q, batch=b) for b in range(4)]
    L = pkg.load_library()

    side = torch.cuda.Stream()           # default priority
    q_in = batches[0].clone()
    out_s = torch.empty(Q, k, dtype=torch.float32, device=DEV)
    out_i = torch.empty(Q, k, dtype=torch.int64, device=DEV)
    torch.cuda.synchronize()
    assert L.ic_index_set_stream(ix.handle, side.cuda_stream) == 0
    with torch.cuda.stream(side):
        ix.search(q_in, k, lam, M, out_s, out_i)       # warm-up outside the capture (one-time kernel attributes)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ix.search(q_in, k, lam, M, out_s, out_i)
    torch.cuda.synchronize()
    assert L.ic_index_set_stream(ix.handle, torch.cuda.current_stream().cuda_stream) == 0

    for r, qb in enumerate(batches):
        want_s, want_i = ix.search(qb, k, lam, M)       # eager, on the current stream
        torch.cuda.synchronize()
        q_in.copy_(qb)
        out_s.fill_(0.0)
        out_i.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_i, want_i), f"replay {r}: ids differ"
        assert torch.equal(out_s, want_s), f"replay {r}: scores differ"
    # a second replay of the last batch, back to back with the first
    graph.replay()
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out_i, want_i) and torch.equal(out_s, want_s)
    del graph
    ix.close()
