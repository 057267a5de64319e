"""The five benchmark configurations at full size, in the launch shape the
benchmark uses, checked on sampled queries.

Masters are generated on the GPU (seeded, see ``workloads``), appended to the
index block by block, and copied to the host block by block for the CPU
reference, which streams them through its chunked scan.  The reference sees
only the fp32 masters; rows needed for the stored-value check are gathered from
the masters and quantised by the reference's own quantiser.
"""
import sys
import time

import numpy as np
import pytest
import torch

import parity
import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
CHUNK = 16 * workloads.BLOCK      # rows per append / host copy


def _say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


class _Run:
    """Builds one configuration on the GPU and the reference lists on the CPU."""

    def __init__(self, pkg, oracle, cfg, sample_q, extra_capacity=0, stop_at=None):
        self.cfg, self.oracle = cfg, oracle
        self.wl = workloads.Workload(cfg, DEV)
        store = pkg.STORE_BF16 if cfg.store == "bf16" else pkg.STORE_FP8_E4M3
        self.ix = pkg.Index(cfg.d, cfg.N + extra_capacity, store, min(cfg.Q, 8192), max(cfg.k, 1), DEV)
        self.E = torch.empty(cfg.N, cfg.d, dtype=torch.float32, device=DEV)
        self.U = torch.empty(cfg.N, dtype=torch.float32, device=DEV) if cfg.util != "none" else None
        self.M = torch.empty(cfg.N, dtype=torch.uint8, device=DEV) if cfg.p_valid < 1 else None
        self.Qd = self.wl.queries(cfg.Q)
        self.Qm = self.Qd.cpu().numpy()
        self.sample_q = list(sample_q)
        self.kk = 4 * cfg.k
        self.scan = oracle.Scan(self.Qm[self.sample_q], self.kk, cfg.lam)
        self.fed = 0
        self.n_valid = 0

    def feed(self, upto, append=True):
        """Generate rows [fed, upto), append them, and stream them through the reference."""
        cfg = self.cfg
        while self.fed < upto:
            n = min(CHUNK, upto - self.fed)
            E, U, M = self.wl.rows(self.fed, n)
            self.E[self.fed:self.fed + n] = E
            if U is not None:
                self.U[self.fed:self.fed + n] = U
            if M is not None:
                self.M[self.fed:self.fed + n] = M
            if append:
                first = self.ix.append(E, U)
                assert first == self.fed
            Mh = None if M is None else M.cpu().numpy()
            self.scan.scan(E.cpu().numpy(), None if U is None else U.cpu().numpy(), Mh)
            self.n_valid += n if Mh is None else int(Mh.sum())
            self.fed += n
            print(f"   fed {self.fed}/{upto}", flush=True)

    def reference(self):
        _, ids, s64 = self.scan.finish()
        return ids, s64

    def check(self, gs, gi, ref, where, sharp=True):
        ref_i, ref_s = ref
        cfg = self.cfg
        gs, gi = gs.cpu().numpy(), gi.cpu().numpy()

        def fetch(ids):
            t = torch.from_numpy(np.asarray(ids)).to(DEV)
            return self.E[t].cpu().numpy(), (None if self.U is None else self.U[t].cpu().numpy())

        def is_valid(ids):
            if self.M is None:
                return np.ones(len(ids), bool)
            return self.M[torch.from_numpy(np.asarray(ids)).to(DEV)].cpu().numpy() != 0

        agg = []
        for j, q in enumerate(self.sample_q):
            if q >= gs.shape[0]:
                continue
            agg.append(parity.check_query(cfg.store, gs[q], gi[q], cfg.k, cfg.lam, self.Qm[q], ref_i[j],
                                          ref_s[j], self.n_valid, fetch, is_valid, f"{where} q={q}",
                                          sharp=sharp))
        print(f"   {where}: recall@k vs fp32 reference {np.mean([a['recall'] for a in agg]):.4f}, "
              f"max |score - fp32 ref| {max(a['max_err'] for a in agg):.2e}, "
              f"max |score - stored-value ref| {max(a['max_err_q'] for a in agg):.2e}", flush=True)


@pytest.fixture(scope="module")
def pkg():
    import paper_2501_12689_amd as p
    p.load_library()
    return p


def _search(run, Q=None, mask=True):
    cfg = run.cfg
    q = run.Qd if Q is None else run.Qd[:Q].contiguous()
    t0 = time.time()
    s, i = run.ix.search(q, cfg.k, cfg.lam, run.M[:len(run.ix)].contiguous() if (mask and run.M is not None) else None)
    torch.cuda.synchronize()
    print(f"   search Q={q.shape[0]} took {1e3 * (time.time() - t0):.2f} ms (incl. launch)", flush=True)
    return s, i


def _tiled_batch_check(pkg, run, ref, where, Qs=(4096,)):
    """The same store searched with batches large enough for the MFMA-tiled scan: a second index
    (max_queries = the largest batch) is filled from the masters on the GPU, the referenced queries
    sit at the front of every batch, and their rows of the result go through the same checks."""
    cfg = run.cfg
    store = pkg.STORE_BF16 if cfg.store == "bf16" else pkg.STORE_FP8_E4M3
    ix2 = pkg.Index(cfg.d, cfg.N, store, max(Qs), cfg.k, DEV)
    for lo in range(0, cfg.N, CHUNK):
        hi = min(cfg.N, lo + CHUNK)
        ix2.append(run.E[lo:hi], None if run.U is None else run.U[lo:hi])
    for Q in Qs:
        big = run.wl.queries(Q, batch=3)
        big[: run.Qd.shape[0]] = run.Qd
        t0 = time.time()
        s, i = ix2.search(big, cfg.k, cfg.lam, run.M)
        torch.cuda.synchronize()
        print(f"   search Q={Q} (tiled) took {1e3 * (time.time() - t0):.2f} ms (incl. launch); "
              f"tiles done again, blocks redone: {ix2.tiled_scan_counts()}", flush=True)
        run.check(s, i, ref, f"{where} Q={Q}")
    ix2.close()


def test_c1_full(pkg, oracle):
    cfg = workloads.C1
    _say(f"{cfg}")
    run = _Run(pkg, oracle, cfg, range(cfg.Q))
    run.feed(cfg.N)
    s, i = _search(run)
    run.check(s, i, run.reference(), "C1")


def test_c2_full(pkg, oracle):
    cfg = workloads.C2
    _say(f"{cfg}")
    run = _Run(pkg, oracle, cfg, range(0, cfg.Q, 16))
    run.feed(cfg.N)
    s, i = _search(run)
    run.check(s, i, run.reference(), "C2")


def test_c3_full(pkg, oracle):
    cfg = workloads.C3
    _say(f"{cfg}")
    run = _Run(pkg, oracle, cfg, [0, 5, 7, 13, 31, 47, 62, 63])
    run.feed(cfg.N)
    ref = run.reference()
    s64, i64 = _search(run)
    run.check(s64, i64, ref, "C3 Q=64")
    for Q in (1, 8):
        s, i = _search(run, Q)
        assert torch.equal(i, i64[:Q]) and torch.equal(s, s64[:Q])
        run.check(s, i, ref, f"C3 Q={Q}")
    _tiled_batch_check(pkg, run, ref, "C3 (tiled)", Qs=(4096,))


def test_c4_full(pkg, oracle):
    cfg = workloads.C4
    _say(f"{cfg}")
    run = _Run(pkg, oracle, cfg, [0, 63, 64, 1000, 2047, 2048, 4000, 4095])
    run.feed(cfg.N)
    s, i = _search(run)
    run.check(s, i, run.reference(), "C4")


def test_c5_full_with_appends(pkg, oracle):
    cfg = workloads.C5
    _say(f"{cfg}")
    run = _Run(pkg, oracle, cfg, [0, 1, 9, 17, 33, 40, 62, 63])
    step = 100_000
    run.feed(cfg.N - 2 * step)
    ref = run.reference()                   # the reference's lists over the rows fed so far
    for Q in (1, 64):
        s, i = _search(run, Q)
        run.check(s, i, ref, f"C5 Q={Q}, {len(run.ix)} rows")
    run.feed(cfg.N - step)                  # append 100k rows between search batches
    s, i = _search(run, 16)
    run.check(s, i, run.reference(), f"C5 Q=16, {len(run.ix)} rows")
    run.feed(cfg.N)
    ref = run.reference()
    s, i = _search(run)
    run.check(s, i, ref, "C5 Q=64")
    for Q in (2, 4, 8, 32):                 # the rest of the streaming half of the sweep
        s2, i2 = _search(run, Q)
        assert torch.equal(i2, i[:Q]) and torch.equal(s2, s[:Q])
    # larger batches on an index made for 64 queries: several passes of 64 queries
    big = workloads.Workload(cfg, DEV).queries(512, batch=1)
    s2, i2 = run.ix.search(big, cfg.k, cfg.lam)
    s3, i3 = run.ix.search(big[100:101].contiguous(), cfg.k, cfg.lam)
    torch.cuda.synchronize()
    assert torch.equal(i2[100], i3[0]) and torch.equal(s2[100], s3[0])
    # the tiled half of the sweep, up to the largest batch the layout allows
    _tiled_batch_check(pkg, run, ref, "C5 (tiled, fp8)", Qs=(128, 256, 512, 1024, 2048, 4096, 8192))


def test_store_of_100_million_short_rows(pkg, oracle):
    """Row ids past 2^26 and a store (row-major and step-major copies) of 12.8 GB each made of 128-byte
    rows, the shortest there are: the tiled scan (256 queries) and the streaming scan (the first 64 of
    them) against the reference on four queries, two of which sit next to the last rows of the store;
    then a tenth of the rows is evicted and squeezed out and the searches are repeated."""
    cfg = workloads.Config("L", N=100_000_001, d=64, clusters=64, Q=256, k=10, store="fp8", zipf=1.1, lam=0.1,
                           util="uniform", p_valid=0.9, seed=126890 + 6)
    _say(f"{cfg}")
    sample = [0, 1, 63, 255]
    run = _Run(pkg, oracle, cfg, sample)
    # queries 0 and 1 are (nearly) the last two rows; the reference gets the same queries
    tail, _, _ = run.wl.rows(cfg.N - 2, 2)
    run.Qd[:2] = tail + 0.01 * run.Qd[:2]
    run.Qm = run.Qd.cpu().numpy()
    run.scan = oracle.Scan(run.Qm[sample], run.kk, cfg.lam)
    run.feed(cfg.N)
    ref = run.reference()
    s, i = _search(run)
    print(f"   tiles done again, blocks redone: {run.ix.tiled_scan_counts()}", flush=True)
    run.check(s, i, ref, "100 M rows, tiled")
    s64, i64 = _search(run, 64)
    run.check(s64, i64, ref, "100 M rows, streaming")
    assert int(i.max()) >= cfg.N - 2 or int(i64.max()) >= cfg.N - 2 or not bool(run.M[cfg.N - 2:].any())
    # evict every tenth row but the sampled queries' neighbours' chances stay as the reference sees them:
    # the reference is run again over the surviving rows
    g = torch.Generator(device=DEV)
    g.manual_seed(6)
    gone = torch.randperm(cfg.N, device=DEV, generator=g)[: cfg.N // 10]
    run.ix.invalidate(gone)
    id_map = run.ix.compact()
    keep = id_map >= 0
    assert int(keep.sum()) == len(run.ix) == cfg.N - gone.numel()
    run.E, run.U, run.M = run.E[keep], run.U[keep], run.M[keep]
    scan2 = oracle.Scan(run.Qm[sample], run.kk, cfg.lam)
    n2 = len(run.ix)
    run.n_valid = 0
    for lo in range(0, n2, CHUNK):
        hi = min(n2, lo + CHUNK)
        Mh = run.M[lo:hi].cpu().numpy()
        scan2.scan(run.E[lo:hi].cpu().numpy(), run.U[lo:hi].cpu().numpy(), Mh)
        run.n_valid += int(Mh.sum())
    _, ids2, s2 = scan2.finish()
    s, i = _search(run)
    run.check(s, i, (ids2, s2), "90 M rows after compaction, tiled")
    s64, i64 = _search(run, 64)
    run.check(s64, i64, (ids2, s2), "90 M rows after compaction, streaming")
