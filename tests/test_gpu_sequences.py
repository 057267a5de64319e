"""GPU parity of whole life cycles: seeded random sequences of appends, utility updates, evictions,
compactions and searches (plain, with a threshold, of stored rows) on one index, through the C ABI,
against a model of the store kept on the CPU with the reference's definitions.

Every test in the other files checks one call after a fixed preparation; these check that the calls
compose: a search after any mix of the others sees exactly the rows, utilities and ids the model says.
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
    return p


class _Model:
    """Masters, utilities and validity of the live rows, in store order."""

    def __init__(self, d):
        self.E = np.zeros((0, d), np.float32)
        self.U = np.zeros(0, np.float32)
        self.V = np.zeros(0, np.uint8)

    def __len__(self):
        return len(self.E)


def _draw_sequence(rng, large):
    """Shape of one sequence.  ``large``: the store is big enough for the tiled scan, most of it arrives
    in the first append, and evictions stay small, so that the later batches of 65 and more queries
    take that path between the maintenance calls."""
    store = "fp8" if rng.random() < 0.4 else "bf16"
    d = int(rng.choice([rng.integers(8, 65), rng.integers(65, 300), rng.integers(300, 700)]))
    if large:
        total = int(rng.choice([rng.integers(280000, 340000), rng.integers(70000, 130000)]))
        max_q = int(rng.choice([200, 300]))
    else:
        total = int(rng.integers(2000, 60000))
        max_q = int(rng.choice([64, 200]))
    total = min(total, int(8e7 // d))
    k = int(rng.choice([1, rng.integers(2, 17), rng.integers(17, 65)]))
    lam = float(rng.choice([0.0, 0.3]))
    ops = ["append"] + [str(rng.choice(["append", "search", "search", "invalidate", "compact", "set_utility",
                                        "scale_utility", "self_search", "threshold"]))
                        for _ in range(int(rng.integers(4, 10)))] + ["search"]
    return store, d, total, max_q, k, lam, ops


@pytest.mark.parametrize("seed,large", [(s, s % 2 == 1) for s in range(7100, 7112)],
                         ids=lambda v: str(v))
def test_random_life_cycle(pkg, oracle, seed, large):
    rng = np.random.default_rng(seed)
    store, d, total, max_q, k, lam, ops = _draw_sequence(rng, large)
    _say(f"life cycle seed={seed} {store} d={d} rows={total} max_queries={max_q} k={k} lambda={lam}: {' '.join(ops)}")
    cfg = workloads.Config("S", N=total, d=d, clusters=int(rng.integers(2, 30)), Q=max_q, k=k, store=store,
                           zipf=1.1, lam=lam, util="uniform", seed=seed)
    wl = workloads.Workload(cfg, "cpu")
    E_all, U_all, _ = wl.rows(0, total)
    E_all, U_all = E_all.numpy(), U_all.numpy()
    sid = pkg.STORE_BF16 if store == "bf16" else pkg.STORE_FP8_E4M3
    ix = pkg.Index(d, total, sid, max_q, 65, DEV)
    m = _Model(d)
    fed = 0                                     # masters handed to append so far
    first = int(total * (rng.uniform(0.95, 0.99) if large else rng.uniform(0.5, 0.9)))
    up = lambda a: torch.from_numpy(a).to(DEV)

    for step, op in enumerate(ops):
        where = f"seed {seed} step {step} {op}"
        if op == "append":
            room = min(total - len(m), total - fed)
            if room <= 0:
                continue
            cnt = min(room, first if fed == 0 else int(rng.integers(1, max(2, room))))
            at = ix.append(up(E_all[fed:fed + cnt]), up(U_all[fed:fed + cnt]))
            assert at == len(m), where
            m.E = np.concatenate([m.E, E_all[fed:fed + cnt]])
            m.U = np.concatenate([m.U, U_all[fed:fed + cnt]])
            m.V = np.concatenate([m.V, np.ones(cnt, np.uint8)])
            fed += cnt
        elif op == "invalidate":
            share = rng.uniform(0.001, 0.03) if large else rng.uniform(0.01, 0.4)
            ids = rng.choice(len(m), max(1, int(len(m) * share)), replace=False).astype(np.int64)
            ix.invalidate(up(ids))
            m.V = oracle.invalidate(m.V, ids)
        elif op == "set_utility":
            ids = rng.choice(len(m), max(1, len(m) // 7), replace=False).astype(np.int64)
            vals = (rng.random(len(ids)) * 2).astype(np.float32)
            ix.set_utility(up(ids), up(vals))
            m.U = oracle.set_utility(m.U, ids, vals)
        elif op == "scale_utility":
            ix.scale_utility(0.9)
            m.U = oracle.scale_utility(m.U, 0.9)
        elif op == "compact":
            id_map = ix.compact().cpu().numpy()
            want, new_n = oracle.compaction_map(m.V)
            assert np.array_equal(id_map, want) and len(ix) == new_n, where
            keep = m.V != 0
            m.E, m.U, m.V = m.E[keep], m.U[keep], np.ones(new_n, np.uint8)
        elif op in ("search", "threshold"):
            Q = int(rng.choice([1, rng.integers(2, 65), rng.integers(65, 129), rng.integers(129, max_q + 190)]))
            Qm = wl.queries(Q, batch=int(rng.integers(0, 1000))).numpy()
            M = (rng.random(len(m)) < 0.8).astype(np.uint8) if rng.random() < 0.4 else None
            visible = m.V if M is None else (m.V & M)
            qd, md = up(Qm), (None if M is None else up(M))
            s, i = ix.search(qd, k, lam, md)
            torch.cuda.synchronize()
            s, i = s.cpu().numpy(), i.cpu().numpy()
            sample = sorted(set([0, Q - 1] + [int(x) for x in rng.integers(0, Q, size=5)]))
            parity.check_batch(store, s, i, m.E, m.U, visible, Qm, k, lam, where, queries=sample)
            if op == "threshold" and np.isfinite(s).any():
                cut = float(np.median(s[np.isfinite(s)]))
                s2, i2, c2 = ix.search_threshold(qd, k, cut, lam, md)
                torch.cuda.synchronize()
                kept = s >= np.float32(cut)      # the same fp32 scores, cut at the threshold
                assert np.array_equal(c2.cpu().numpy(), kept.sum(1)), where
                assert np.array_equal(i2.cpu().numpy(), np.where(kept, i, -1)), where
        elif op == "self_search" and len(m) > 300 and m.V.all():
            cnt = int(rng.choice([5, 64, 200]))
            first_row = int(rng.integers(0, len(m) - cnt))
            kk = min(k, 32)
            s, i = ix.self_search(first_row, cnt, kk, lam)
            torch.cuda.synchronize()
            s, i = s.cpu().numpy(), i.cpu().numpy()
            for r in (0, cnt - 1):
                assert first_row + r not in i[r], f"{where}: row {first_row + r} returned itself"
                others = np.ones(len(m), np.uint8)
                others[first_row + r] = 0
                parity.check_batch(store, s[r:r + 1], i[r:r + 1], m.E, m.U, others, m.E[first_row + r][None],
                                   kk, lam, f"{where} row {r}")
    ix.close()
