"""CPU tests: the comparison rules themselves, the host logic of the C ABI, and
that the built library exports what the header declares."""
import ctypes
import os
import re

import numpy as np
import pytest

import parity
import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _case(store="bf16", N=3000, Q=6, k=12, seed=0):
    cfg = workloads.C2.scaled(N=N, Q=Q, k=k, d=96, clusters=16, seed=seed, store=store)
    wl = workloads.Workload(cfg, "cpu")
    E, U, M = (t.numpy() if t is not None else None for t in wl.rows(0, N))
    return cfg, E, U, M, wl.queries().numpy()


def _stored_value_result(oracle, store, E, U, M, Qm, k, lam):
    """What a correct index returns: the reference run on the reference's own quantised values."""
    if store == "bf16":
        e = oracle.decode_bf16(oracle.quantize_bf16(E))
        q = oracle.decode_bf16(oracle.quantize_bf16(Qm))
        s32, ids, _ = oracle.search(e, q, k, lam, U, M, normalize=False)
    else:
        ce, se = oracle.quantize_fp8(E)
        cq, sq = oracle.quantize_fp8(Qm)
        s32, ids, _ = oracle.search(oracle.decode_e4m3(ce), oracle.decode_e4m3(cq), k, lam, U, M,
                                    normalize=False, row_scale=se, q_scale=sq)
    return s32, ids


@pytest.mark.parametrize("store", ["bf16", "fp8"])
def test_checker_accepts_reference_on_stored_values(oracle, store):
    cfg, E, U, M, Qm = _case(store)
    s32, ids = _stored_value_result(oracle, store, E, U, M, Qm, cfg.k, cfg.lam)
    st = parity.check_batch(store, s32, ids, E, U, M, Qm, cfg.k, cfg.lam, "self")
    assert st["max_err_q"] < 1e-6 and st["max_err"] < parity.TAU[store]


def test_checker_rejects_planted_mistakes(oracle):
    cfg, E, U, M, Qm = _case("bf16")
    s32, ids = _stored_value_result(oracle, "bf16", E, U, M, Qm, cfg.k, cfg.lam)
    far = oracle.search(E, Qm, cfg.k * 20, cfg.lam, U, M)[1]

    bad_i = ids.copy(); bad_i[2, 3] = far[2, -1]                 # a far worse example slipped in
    with pytest.raises(AssertionError):
        parity.check_batch("bf16", s32, bad_i, E, U, M, Qm, cfg.k, cfg.lam, "swap")
    bad_s = s32.copy(); bad_s[1] += 3e-4; bad_s[1] = np.sort(bad_s[1])[::-1]   # score drift > tau_q
    with pytest.raises(AssertionError):
        parity.check_batch("bf16", bad_s, ids, E, U, M, Qm, cfg.k, cfg.lam, "drift")
    masked = np.flatnonzero(M == 0)
    bad_i = ids.copy(); bad_i[0, -1] = masked[0]                 # a masked row returned
    with pytest.raises(AssertionError):
        parity.check_batch("bf16", s32, bad_i, E, U, M, Qm, cfg.k, cfg.lam, "masked")
    bad_i = ids.copy(); bad_i[4, 5] = bad_i[4, 4]                # duplicate id
    with pytest.raises(AssertionError):
        parity.check_batch("bf16", s32, bad_i, E, U, M, Qm, cfg.k, cfg.lam, "dup")
    bad_i = ids.copy(); bad_s = s32.copy()                       # rows swapped: order broken
    bad_i[3, [0, 1]] = bad_i[3, [1, 0]]; bad_s[3, [0, 1]] = bad_s[3, [1, 0]]
    with pytest.raises(AssertionError):
        parity.check_batch("bf16", bad_s, bad_i, E, U, M, Qm, cfg.k, cfg.lam, "order")
    # reference without the utility term: caught by the band/sharp rules
    s0, i0 = _stored_value_result(oracle, "bf16", E, None, M, Qm, cfg.k, 0.0)
    with pytest.raises(AssertionError):
        parity.check_batch("bf16", s0, i0, E, U, M, Qm, cfg.k, cfg.lam, "no-utility")


# ------------------------------------------------------------------ C ABI, host side

def _header_functions():
    txt = open(os.path.join(ROOT, "include", "iccache.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(ic_[a-z_0-9]+)\s*\(", txt)))


def test_library_exports_every_declared_symbol():
    import paper_2501_12689_amd as pkg
    L = pkg.load_library()
    names = _header_functions()
    assert {"ic_index_create", "ic_index_append", "ic_search", "ic_index_destroy"} <= set(names)
    for n in names:
        assert hasattr(L, n), f"{n} declared in iccache.h but not exported"
    from paper_2501_12689_amd import binding
    assert set(binding.EXPORTS) == set(names)


def test_workspace_bytes_arithmetic():
    import paper_2501_12689_amd as pkg
    w = pkg.ic_workspace_bytes
    M = 1 << 20                       # capacities are padded to whole 256-row tiles
    base = w(768, pkg.STORE_BF16, M, 64, 64)
    more = w(768, pkg.STORE_BF16, 2 * M, 64, 64)
    # M more rows: 1536 B row + 4 B utility + 4 B score bias + 4 B sharing domain + 1 B validity each, and 8 B of
    # compaction scratch per 1024 rows (up to alignment)
    assert abs((more - base) - M * (1536 + 4 + 4 + 4 + 1) - M // 1024 * 8) <= 1024
    f8 = w(1024, pkg.STORE_FP8_E4M3, 2 * M, 64, 64) - w(1024, pkg.STORE_FP8_E4M3, M, 64, 64)
    assert abs(f8 - M * (1024 + 4 + 4 + 4 + 4 + 1) - M // 1024 * 8) <= 1024      # + per-row scale
    # large batches add the per-query candidate lists of the tiled scan
    assert w(768, pkg.STORE_BF16, M, 4096, 16) > w(768, pkg.STORE_BF16, M, 64, 16) + 4096 * 2048 * 8
    # rows pad to 128 B: d = 100 bf16 -> 256 B
    a = w(100, pkg.STORE_BF16, 1 << 20, 64, 64) - w(100, pkg.STORE_BF16, 1 << 19, 64, 64)
    assert abs(a - (1 << 19) * (256 + 4 + 4 + 4 + 1) - (1 << 9) * 8) <= 1024
    for bad in [(0, 0, 10, 1, 1), (1025, 0, 10, 1, 1), (2049, 1, 10, 1, 1), (64, 2, 10, 1, 1),
                (64, 0, 0, 1, 1), (64, 0, 10, 0, 1), (64, 0, 10, 1, 0), (64, 0, 10, 1, 129)]:
        assert w(*bad) == 0, bad


def test_status_codes_without_a_gpu():
    """Argument errors are decided on the host before any launch."""
    import paper_2501_12689_amd as pkg
    L = pkg.load_library()
    need = pkg.ic_workspace_bytes(64, pkg.STORE_BF16, 100, 8, 16)
    h = ctypes.c_void_p()
    fake = ctypes.c_void_p(1 << 20)          # aligned, never dereferenced by these calls
    assert L.ic_index_create(None, 64, 0, 100, 8, 16, fake, need, None) == 1
    assert L.ic_index_create(ctypes.byref(h), 64, 0, 100, 8, 16, None, need, None) == 1
    assert L.ic_index_create(ctypes.byref(h), 64, 0, 100, 8, 16, ctypes.c_void_p((1 << 20) + 8), need, None) == 1
    assert L.ic_index_create(ctypes.byref(h), 64, 0, 100, 8, 16, fake, need - 1, None) == 3
    assert L.ic_index_create(ctypes.byref(h), 64, 7, 100, 8, 16, fake, need, None) == 1
    assert L.ic_index_create(ctypes.byref(h), 64, 0, 100, 8, 16, fake, need, None) == 0
    assert L.ic_index_size(h) == 0 and L.ic_index_size(None) == -1
    first = ctypes.c_int64(-5)
    assert L.ic_index_append(h, fake, None, 101, ctypes.byref(first)) == 3     # beyond capacity
    assert L.ic_index_append(h, None, None, 5, None) == 1
    assert L.ic_index_append(h, fake, None, -1, None) == 1
    assert L.ic_index_append(h, None, None, 0, ctypes.byref(first)) == 0 and first.value == 0
    assert L.ic_search(h, fake, 4, 0, 0.0, None, fake, fake) == 1              # k < 1
    assert L.ic_search(h, fake, 4, 17, 0.0, None, fake, fake) == 1             # k > max_k
    assert L.ic_search(h, fake, -1, 4, 0.0, None, fake, fake) == 1
    assert L.ic_search(h, None, 4, 4, 0.0, None, fake, fake) == 1
    assert L.ic_search(h, fake, 4, 4, 0.0, None, None, fake) == 1
    assert L.ic_search(h, None, 0, 4, 0.0, None, None, None) == 0              # Q == 0: no-op
    assert L.ic_search(None, fake, 4, 4, 0.0, None, fake, fake) == 1
    assert L.ic_index_size(h) == 0
    # maintenance calls: argument errors, and no-ops on an empty index (nothing is launched)
    assert L.ic_index_set_utility(None, fake, fake, 1) == 1 and L.ic_index_set_utility(h, None, fake, 1) == 1
    assert L.ic_index_set_utility(h, fake, None, 1) == 1 and L.ic_index_set_utility(h, fake, fake, -1) == 1
    assert L.ic_index_set_utility(h, None, None, 0) == 0
    assert L.ic_index_scale_utility(None, ctypes.c_float(0.9)) == 1 and L.ic_index_scale_utility(h, ctypes.c_float(0.9)) == 0
    assert L.ic_index_invalidate(None, fake, 1) == 1 and L.ic_index_invalidate(h, None, 1) == 1
    assert L.ic_index_invalidate(h, None, 0) == 0
    assert L.ic_index_set_domains(None, fake, fake, 1) == 1 and L.ic_index_set_domains(h, fake, None, 1) == 1
    assert L.ic_index_set_domains(h, None, None, 0) == 0
    assert L.ic_search_domains(h, fake, 4, 4, 0.0, None, None, fake, fake) == 1   # no query domains
    assert L.ic_search_domains(h, None, 0, 4, 0.0, None, None, None, None) == 0   # Q == 0: no-op
    again, redone = ctypes.c_int64(-1), ctypes.c_int64(-1)
    assert L.ic_index_tiled_scan_counts(None, ctypes.byref(again), ctypes.byref(redone)) == 1
    # no large batch has run: zeros, and no device is touched
    assert L.ic_index_tiled_scan_counts(h, ctypes.byref(again), ctypes.byref(redone)) == 0
    assert again.value == 0 and redone.value == 0
    assert L.ic_index_tiled_scan_counts(h, None, None) == 0
    left = ctypes.c_int64(-7)
    assert L.ic_index_compact(None, fake, None) == 1 and L.ic_index_compact(h, None, None) == 1
    assert L.ic_index_compact(h, fake, ctypes.byref(left)) == 0 and left.value == 0
    # cluster pruning: sizes and argument errors are host arithmetic as well
    assert L.ic_ivf_workspace_bytes(None, 10, 4) == 0 and L.ic_ivf_workspace_bytes(h, 0, 4) == 0
    assert L.ic_ivf_workspace_bytes(h, 10, 0) == 0 and L.ic_ivf_workspace_bytes(h, 10, 129) == 0
    need_ivf = L.ic_ivf_workspace_bytes(h, 10, 4)
    assert need_ivf > 2 * need                     # a centroid index and a sorted copy of the store
    v = ctypes.c_void_p()
    assert L.ic_ivf_create(None, h, 10, 4, fake, need_ivf) == 1 and L.ic_ivf_create(ctypes.byref(v), None, 10, 4, fake, need_ivf) == 1
    assert L.ic_ivf_create(ctypes.byref(v), h, 10, 4, fake, need_ivf - 1) == 3
    assert L.ic_ivf_create(ctypes.byref(v), h, 10, 4, fake, need_ivf) == 0
    assert L.ic_ivf_search(v, fake, 1, 1, 1, 0.0, fake, fake) == 1          # no centroids, no lists yet
    assert L.ic_ivf_assign(v) == 1 and L.ic_ivf_update_centroids(v) == 1    # no centroids yet
    assert L.ic_ivf_train(v, 1) == 1                                         # empty base index
    assert L.ic_ivf_destroy(v) == 0 and L.ic_ivf_destroy(None) == 1
    assert L.ic_status_string(3) == b"capacity exceeded"
    assert L.ic_index_destroy(h) == 0 and L.ic_index_destroy(None) == 1


def test_workload_generator_properties():
    """Inputs have the stated structure: unit rows, clustered, Zipf head, mask/utility rates."""
    import torch
    cfg = workloads.C3.scaled(N=40000, clusters=64, d=64)
    wl = workloads.Workload(cfg, "cpu")
    E, U, M = wl.rows(0, cfg.N)
    assert U is None and M is None
    assert torch.allclose(E.norm(dim=1), torch.ones(cfg.N), atol=1e-5)
    sims = E @ wl.centres.T
    best = sims.max(1).values
    assert abs(float(best.mean()) - 1 / (1 + cfg.sigma ** 2) ** 0.5) < 0.02
    counts = torch.bincount(sims.argmax(1), minlength=64).double()
    w = torch.arange(1, 65, dtype=torch.float64) ** -1.1
    assert abs(float(counts[0] / cfg.N) - float(w[0] / w.sum())) < 0.01
    # any sub-range regenerates identically
    E2, _, _ = wl.rows(65000, 700)
    full = wl.rows(64000, 3000)[0]
    assert torch.equal(full[1000:1700], E2)
    c4 = workloads.C4.scaled(N=50000, clusters=8, d=32)
    _, U4, M4 = workloads.Workload(c4, "cpu").rows(0, c4.N)
    assert abs(float(U4.mean()) - 2 / 7) < 0.01 and abs(float(M4.float().mean()) - 0.9) < 0.01
