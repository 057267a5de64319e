#!/usr/bin/env python3
"""Benchmark: top-k example retrieval throughput on one MI355X.

Workload: the N = 10,000,000, d = 768 bf16 configuration (4096-cluster Zipf
mixture, k = 64, lambda = 0, no mask), query batches of 1, 8 and 64.  A step is
one ``ic_search`` call on a batch that is already resident in HBM: query
preparation, similarity + score epilogue + per-slice partial top-k, cross-slice
merge.  The headline value is queries/s at Q = 64; Q = 1 and Q = 8 are reported
in ``config.per_Q``.  Appending (normalise + quantise + store) happens once per
example, not per batch; its rate is reported separately under ``append``.

The matrix-core regime is timed as well (fewer steps, they are long): Q = 4096 on
the same store (``config.per_Q["4096"]``) and the N = 4,000,000, d = 1024, k = 16
configuration with utility and mask (``large_batch``, ``roofline_mfma``); and the fp8 store
(N = 20,000,000, d = 1024, k = 100, built by appends of 100,000 rows) with Q swept over the powers of
two from 1 to 8192, 100,000 more rows appended (and timed) before every batch size after the first
(``fp8_store``: both roofline fractions per Q).  ``maintenance`` times the eviction of the masked rows of the d = 1024
configuration and the compaction that squeezes them out; ``census`` runs a self-search of every
row of a 1,000,000-row store against all the others; ``cluster_pruning`` trains K = sqrt(N)
clusters on the headline store and times the pruned search, with its recall against the exact one.

Prints one JSON line.  ``roofline`` refers to the scan kernel, timed with HIP
events on the library's stream inside the timed steps; ``cpu_baseline`` is the
CPU reference timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
MFMA_FP8_PEAK_TFLOPS = 5000.0
# HBM bytes per launch of the two dominant kernels, from two rocprofv3 counter runs of this program
# (FETCH_SIZE and WRITE_SIZE in KiB per dispatch, each scaled by what the same counter reads for a plain
# 1 GiB copy: 1,048,576 / 524,300 and 1.0).  Valid for the kernels as committed with the rocprofv3
# summaries of these runs; set to None when a kernel changes until its counters are taken again.
SCAN_TRAFFIC_BYTES_Q64 = (7_502_488 * (1_048_576 / 524_300) + 3_526) * 1024      # scan_stream, N = 10M, d = 768, Q = 64
GEMM_TRAFFIC_BYTES_C4 = (23_786_629 * (1_048_576 / 524_300) + 225_161) * 1024    # scan_gemm, N = 4M, d = 1024, Q = 4096
LARGE_Q = 4096


def time_search(ix, torch, qd, k, lam, mask, out_s, out_i, warmup, steps):
    """Time `steps` searches on resident inputs.

    Returns (ms per step = whole timed region / steps, scan kernel ms per launch, wall ms per step,
    {median, p10, p90} of the single steps from an event recorded after every step)."""
    ix.set_timing(False)
    for _ in range(warmup):
        ix.search(qd, k, lam, mask, out_s, out_i)
    torch.cuda.synchronize()
    ix.set_timing(True)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    # the library brackets every scan launch with events on this stream; nothing waits
    for i in range(steps):
        ix.search(qd, k, lam, mask, out_s, out_i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    scan_ms, launches = ix.scan_time_ms()
    ix.set_timing(False)
    each = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
    pick = lambda f: each[min(steps - 1, int(f * steps))]
    spread = {"median": pick(0.5), "p10": pick(0.1), "p90": pick(0.9)}
    return ev[0].elapsed_time(ev[steps]) / steps, scan_ms / max(launches, 1), wall_ms / steps, spread


def graph_replay_ms(pkg, torch, ix, qd, k, lam, mask, out_s, out_i, steps):
    """The same search captured once into a HIP graph on a side stream and replayed `steps` times:
    what a launch-bound small cache gains when the caller takes the launches off the host."""
    L = pkg.load_library()
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    L.ic_index_set_stream(ix.handle, side.cuda_stream)
    with torch.cuda.stream(side):
        ix.search(qd, k, lam, mask, out_s, out_i)    # one-time kernel attributes are set outside the capture
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ix.search(qd, k, lam, mask, out_s, out_i)
    torch.cuda.synchronize()
    L.ic_index_set_stream(ix.handle, torch.cuda.current_stream().cuda_stream)
    for _ in range(5):
        graph.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    del graph
    return e0.elapsed_time(e1) / steps


def say(msg: str) -> None:
    """Progress line on stderr (stdout carries only the JSON line)."""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def cluster_pruning_leg(pkg, torch, np, ix, wl, cfg, Q, k, probes):
    """K = sqrt(N) clusters by two K-Means iterations on the index, then the pruned search at several
    numbers of probed clusters: time per batch and recall against the exact search."""
    qd = wl.queries(Q, batch=Q)
    exact_s, exact_i = ix.search(qd, k, cfg.lam)
    K = max(1, int(round(len(ix) ** 0.5)))
    ivf = pkg.Ivf(ix, K, max(probes))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ivf.train(2)
    torch.cuda.synchronize()
    leg = {"N": len(ix), "K": K, "kmeans_iterations": 2, "train_s": time.perf_counter() - t0, "Q": Q, "k": k,
           "per_nprobe": {}}
    sizes = ivf.view()[1].diff()                     # rows per cluster list
    for nprobe in probes:
        # comparisons per query against the paper's cost model K + N/K (times the lists probed)
        scanned = float(sizes[ivf.probed_clusters(qd, nprobe)].sum(1).double().mean())
        for _ in range(3):
            ivf.search(qd, k, nprobe, cfg.lam)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            s_, i_ = ivf.search(qd, k, nprobe, cfg.lam)
        e1.record()
        e1.synchronize()
        ms = e0.elapsed_time(e1) / 20
        a, b = i_.cpu().numpy(), exact_i.cpu().numpy()
        rec = float(np.mean([len(set(a[q].tolist()) & set(b[q].tolist()) - {-1}) / max(1, int((b[q] >= 0).sum()))
                             for q in range(Q)]))
        leg["per_nprobe"][str(nprobe)] = {"ms_per_step": ms, "queries_per_s": Q / (ms * 1e-3),
                                          f"recall_at_{k}_vs_exact": rec,
                                          "comparisons_per_query": K + scanned,
                                          "cost_model_K_plus_nprobe_N_over_K": K + nprobe * len(ix) / K,
                                          "exact_scan_comparisons": len(ix)}
    # every queued launch has finished before the structure's arena is released
    torch.cuda.synchronize()
    ivf.close()
    ivf.arena = None
    return leg


def host_cpu() -> str:
    """Model name and logical CPU count of the host the CPU reference is timed on."""
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for ln in f:
                if ln.lower().startswith("model name"):
                    model = ln.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return f"{model}, {os.cpu_count()} logical CPUs visible"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--rows", type=int, default=None, help="override N (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-large-batch", action="store_true", help="skip the Q = 4096 legs")
    ap.add_argument("--no-fp8", action="store_true", help="skip the fp8 (N = 20M) legs")
    ap.add_argument("--no-cluster-pruning", action="store_true",
                    help="skip the cluster-pruning leg (tens of thousands of small launches while training)")
    ap.add_argument("--no-graph-replay", action="store_true",
                    help="skip the HIP-graph replay timing of the small configurations")
    ap.add_argument("--fp8-sweep", type=str, default=None,
                    help="comma-separated batch sizes of the fp8 leg (default: every power of two from 1 to 8192)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies, so that a counter run over this "
                         "command holds a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2501_12689_amd as pkg
    import workloads

    pkg.load_library()                      # raises if the HIP library is missing: no fallback
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = "cuda:0"
    cfg = workloads.C3 if args.rows is None else workloads.C3.scaled(N=args.rows)
    wl = workloads.Workload(cfg, dev)

    if args.copy_calibration:
        x = torch.full((1 << 28,), 1.0, dtype=torch.float32, device=dev)   # 1 GiB
        y = torch.empty_like(x)
        for _ in range(3):
            y.copy_(x)
        torch.cuda.synchronize()
        del x, y
        torch.cuda.empty_cache()

    # the first launch from the library loads its code object (tens of milliseconds, once per process):
    # a throw-away index takes that, so that the timed appends below measure appends
    warm = pkg.Index(cfg.d, 1024, pkg.STORE_BF16, 64, cfg.k, dev)
    warm.append(torch.zeros(1024, cfg.d, dtype=torch.float32, device=dev), None)
    torch.cuda.synchronize()
    warm.close()
    del warm

    # ---- build the index (timed separately: a1 runs once per example)
    ix = pkg.Index(cfg.d, cfg.N, pkg.STORE_BF16, 64 if args.no_large_batch else LARGE_Q, cfg.k, dev)
    chunk = 16 * workloads.BLOCK
    append_ms, sample_parts = 0.0, []
    sample_n = 0 if args.no_cpu_baseline else min(cfg.N, 6 * chunk)   # rows the CPU baseline scans (about 10 s)
    for lo in range(0, cfg.N, chunk):
        n = min(chunk, cfg.N - lo)
        E, U, M = wl.rows(lo, n)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ix.append(E, U)
        e1.record()
        e1.synchronize()
        append_ms += e0.elapsed_time(e1)
        if lo < sample_n:
            sample_parts.append(E[: max(0, min(n, sample_n - lo))].cpu().numpy())
        del E
    row_bytes = ix.store_view()[0].shape[1]
    store_bytes = cfg.N * row_bytes

    say(f"index built: {cfg.N} rows")
    # ---- timed searches
    per_q = {}
    headline = None
    for Q in (1, 8, 64):
        qd = wl.queries(Q, batch=Q)
        out_s = torch.empty(Q, cfg.k, dtype=torch.float32, device=dev)
        out_i = torch.empty(Q, cfg.k, dtype=torch.int64, device=dev)
        ms, scan, wall, spread = time_search(ix, torch, qd, cfg.k, cfg.lam, None, out_s, out_i, args.warmup, args.steps)
        per_q[str(Q)] = {
            "queries_per_s": Q / (ms * 1e-3),
            "ms_per_step": ms,
            "scan_kernel_ms": scan,
            "scan_GBps": store_bytes / (scan * 1e-3) / 1e9,
            "hbm_frac": store_bytes / (scan * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "wall_ms_per_step": wall, "step_ms": spread,
        }
        if Q == 64:
            headline = per_q[str(Q)]

    say("small batches done")
    # ---- matrix-core regime: Q = 4096 on the same store, then the N = 4M, d = 1024 configuration
    large, roof_mfma, maintenance = None, None, None
    if not args.no_large_batch:
        lsteps, lwarm = max(3, min(10, args.steps)), 2
        Q = LARGE_Q
        qd = wl.queries(Q, batch=Q)
        out_s = torch.empty(Q, cfg.k, dtype=torch.float32, device=dev)
        out_i = torch.empty(Q, cfg.k, dtype=torch.int64, device=dev)
        ms, scan, wall, spread = time_search(ix, torch, qd, cfg.k, cfg.lam, None, out_s, out_i, lwarm, lsteps)
        flop = 2.0 * Q * cfg.N * cfg.d
        per_q[str(Q)] = {
            "queries_per_s": Q / (ms * 1e-3), "ms_per_step": ms, "steps": lsteps, "scan_kernel_ms": scan,
            "scan_TFLOPs": flop / (scan * 1e-3) / 1e12,
            "mfma_frac": flop / (scan * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "step_TFLOPs": flop / (ms * 1e-3) / 1e12, "wall_ms_per_step": wall, "step_ms": spread,
            "tiles_again_blocks_redone": list(ix.tiled_scan_counts()),
        }
        del qd, out_s, out_i
        # batches between the two regimes (one and two query blocks of the tiled scan)
        for Qm in (128, 512):
            qd = wl.queries(Qm, batch=Qm)
            out_s = torch.empty(Qm, cfg.k, dtype=torch.float32, device=dev)
            out_i = torch.empty(Qm, cfg.k, dtype=torch.int64, device=dev)
            ms, scan, wall, spread = time_search(ix, torch, qd, cfg.k, cfg.lam, None, out_s, out_i, lwarm, lsteps)
            flop = 2.0 * Qm * cfg.N * cfg.d
            per_q[str(Qm)] = {
                "queries_per_s": Qm / (ms * 1e-3), "ms_per_step": ms, "steps": lsteps, "scan_kernel_ms": scan,
                "scan_GBps": store_bytes / (scan * 1e-3) / 1e9,
                "hbm_frac": store_bytes / (scan * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "scan_TFLOPs": flop / (scan * 1e-3) / 1e12,
                "mfma_frac": flop / (scan * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                "step_ms": spread, "tiles_again_blocks_redone": list(ix.tiled_scan_counts()),
            }
            del qd, out_s, out_i
    say("Q=4096 on the headline store done")
    # ---- cluster pruning on the same store: K = sqrt(N) clusters, two K-Means iterations
    ivf_leg = None
    if not args.no_large_batch and not args.no_cluster_pruning:
        ivf_leg = cluster_pruning_leg(pkg, torch, np, ix, wl, cfg, 64, cfg.k, (1, 8, 32))
    ix.close()
    ix.arena = None
    del ix
    torch.cuda.empty_cache()
    say("cluster pruning done")
    if not args.no_large_batch:
        c4 = workloads.C4 if args.rows is None else workloads.C4.scaled(N=min(workloads.C4.N, args.rows))
        wl4 = workloads.Workload(c4, dev)
        ix4 = pkg.Index(c4.d, c4.N, pkg.STORE_BF16, c4.Q, c4.k, dev)
        masks = []
        for lo in range(0, c4.N, chunk):
            n = min(chunk, c4.N - lo)
            E, U, M = wl4.rows(lo, n)
            ix4.append(E, U)
            masks.append(M)
            del E
        mask4 = torch.cat(masks) if masks[0] is not None else None
        qd = wl4.queries(c4.Q)
        out_s = torch.empty(c4.Q, c4.k, dtype=torch.float32, device=dev)
        out_i = torch.empty(c4.Q, c4.k, dtype=torch.int64, device=dev)
        ms, scan, wall, spread = time_search(ix4, torch, qd, c4.k, c4.lam, mask4, out_s, out_i, lwarm, lsteps)
        flop = 2.0 * c4.Q * c4.N * c4.d
        large = {
            "workload": f"C4: N={c4.N} d={c4.d} bf16 store, {c4.clusters}-cluster mixture, Q={c4.Q}, k={c4.k}, "
                        f"lambda={c4.lam}, {1.0 - c4.p_valid:.0%} masked rows",
            "queries_per_s": c4.Q / (ms * 1e-3), "ms_per_step": ms, "steps": lsteps, "warmup": lwarm,
            "scan_kernel_ms": scan, "step_TFLOPs": flop / (ms * 1e-3) / 1e12, "wall_ms_per_step": wall,
            "step_ms": spread, "tiles_again_blocks_redone": list(ix4.tiled_scan_counts()),
        }
        ach = flop / (scan * 1e-3) / 1e12
        roof_mfma = {
            "bound": "mfma", "kernel": f"scan_gemm (bf16 MFMA contraction + fused threshold selection), Q={c4.Q}",
            "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS,
            "traffic": GEMM_TRAFFIC_BYTES_C4 if args.rows is None else None, "algorithmic_flops_per_launch": flop,
        }
        # store maintenance on the same index: evict the masked rows for good, squeeze them out,
        # search the smaller store without a mask
        if mask4 is not None:
            gone = torch.nonzero(mask4 == 0).flatten()
            ix4.invalidate(gone)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ix4.compact()
            e1.record()
            e1.synchronize()
            cms = e0.elapsed_time(e1)
            row4 = ix4.store_view()[0].shape[1]
            # every row read once, every survivor written once, and once more into the step-major copy
            moved = c4.N * (row4 + 4) + len(ix4) * (2 * row4 + 4)
            ms2, scan2, _, _ = time_search(ix4, torch, qd, c4.k, c4.lam, None, out_s, out_i, lwarm, lsteps)
            maintenance = {
                "evicted_rows": int(gone.numel()), "rows_left": len(ix4), "compact_ms": cms,
                "compact_rows_per_s": c4.N / (cms * 1e-3),
                "compact_GBps_algorithmic": moved / (cms * 1e-3) / 1e9,
                "compact_hbm_frac": moved / (cms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "search_after_compact": {"queries_per_s": c4.Q / (ms2 * 1e-3), "ms_per_step": ms2,
                                         "scan_kernel_ms": scan2},
            }
        ix4.close()
        ix4.arena = None
        del ix4, mask4, masks, qd, out_s, out_i
        torch.cuda.empty_cache()

    say("large-batch configuration and maintenance done")
    # ---- the two small configurations at their own shapes (report only: C1 fits the last-level
    # cache and is bound by launches; C2 sits at the ridge between the two bounds)
    small_cfgs = None
    if not args.no_large_batch:
        small_cfgs = {}
        for name in ("C1", "C2"):
            cs = workloads.CONFIGS[name]
            if args.rows is not None:
                cs = cs.scaled(N=min(cs.N, args.rows))
            wls = workloads.Workload(cs, dev)
            ixs = pkg.Index(cs.d, cs.N, pkg.STORE_BF16, cs.Q, cs.k, dev)
            masks = []
            for lo in range(0, cs.N, chunk):
                n = min(chunk, cs.N - lo)
                E, U, M = wls.rows(lo, n)
                ixs.append(E, U)
                masks.append(M)
                del E
            mask_s = torch.cat(masks) if masks[0] is not None else None
            qd = wls.queries(cs.Q)
            out_s = torch.empty(cs.Q, cs.k, dtype=torch.float32, device=dev)
            out_i = torch.empty(cs.Q, cs.k, dtype=torch.int64, device=dev)
            ms, scan, wall, spread = time_search(ixs, torch, qd, cs.k, cs.lam, mask_s, out_s, out_i, 5, 50)
            rb = ixs.store_view()[0].shape[1]
            small_cfgs[name] = {
                "workload": f"{name}: N={cs.N} d={cs.d} bf16 store, Q={cs.Q}, k={cs.k}, lambda={cs.lam}, "
                            f"{1.0 - cs.p_valid:.0%} masked rows",
                "queries_per_s": cs.Q / (ms * 1e-3), "ms_per_step": ms, "scan_kernel_ms": scan, "step_ms": spread,
                "step_hbm_frac": cs.N * rb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "step_mfma_frac": 2.0 * cs.Q * cs.N * cs.d / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            }
            if not args.no_graph_replay:
                gms = graph_replay_ms(pkg, torch, ixs, qd, cs.k, cs.lam, mask_s, out_s, out_i, 50)
                small_cfgs[name]["graph_replay"] = {"ms_per_step": gms, "queries_per_s": cs.Q / (gms * 1e-3)}
            if name == "C2" and not args.no_cluster_pruning:
                # the same pruning on a store whose clusters are equally likely (no dominant blob);
                # evicted rows are in no list, so the mask's rows are invalidated first
                if mask_s is not None:
                    ixs.invalidate(torch.nonzero(mask_s == 0).flatten())
                small_cfgs[name]["cluster_pruning"] = cluster_pruning_leg(pkg, torch, np, ixs, wls, cs, 64, cs.k, (1, 4, 16))
            ixs.close()
            ixs.arena = None
            del ixs, qd, out_s, out_i, masks, mask_s
            torch.cuda.empty_cache()
        say("small configurations done")
    # ---- self-similarity census: every row of a 1M-row store against all the others, k = 1
    census = None
    if not args.no_large_batch:
        c2 = workloads.C2 if args.rows is None else workloads.C2.scaled(N=min(workloads.C2.N, args.rows))
        wl2 = workloads.Workload(c2, dev)
        ix2 = pkg.Index(c2.d, c2.N, pkg.STORE_BF16, LARGE_Q, 2, dev)
        for lo in range(0, c2.N, chunk):
            n = min(chunk, c2.N - lo)
            E, U, M = wl2.rows(lo, n)
            ix2.append(E, None)
            del E
        ix2.self_search(0, min(c2.N, 2 * LARGE_Q), 1)          # warm-up
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        top_s, top_i = ix2.self_search(0, c2.N, 1)
        e1.record()
        e1.synchronize()
        cms = e0.elapsed_time(e1)
        flop = 2.0 * c2.N * c2.N * c2.d
        census = {
            "workload": f"self-search of all N={c2.N} rows (d={c2.d} bf16, {c2.clusters}-cluster mixture), k=1, "
                        "each row left out of its own result",
            "ms": cms, "rows_per_s": c2.N / (cms * 1e-3), "TFLOPs": flop / (cms * 1e-3) / 1e12,
            "mfma_frac": flop / (cms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "share_with_a_neighbour_above_0.8": float((top_s[:, 0] > 0.8).float().mean()),
        }
        ix2.close()
        ix2.arena = None
        del ix2, top_s, top_i
        torch.cuda.empty_cache()

    say("census done")
    # ---- fp8 store: N = 20M, d = 1024, k = 100 (built by appends of 100,000 rows), Q = 1, 64, 4096
    fp8 = None
    if not args.no_large_batch and not args.no_fp8:
        c5 = workloads.C5 if args.rows is None else workloads.C5.scaled(N=min(workloads.C5.N, args.rows))
        wl5 = workloads.Workload(c5, dev)
        sweep = [1 << e for e in range(14)]                      # Q = 1 .. 8192
        if args.fp8_sweep:
            sweep = sorted(int(x) for x in args.fp8_sweep.split(","))
        step_rows = 100_000                                       # rows appended between search batches
        ix5 = pkg.Index(c5.d, c5.N + len(sweep) * step_rows, pkg.STORE_FP8_E4M3, max(64, sweep[-1]), c5.k, dev)
        app_ms, app_rows = 0.0, 0

        def timed_append(E):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ix5.append(E, None)
            e1.record()
            e1.synchronize()
            return e0.elapsed_time(e1)

        for lo in range(0, c5.N, chunk):
            n = min(chunk, c5.N - lo)
            E, U, M = wl5.rows(lo, n)
            for a0 in range(0, n, step_rows):
                a1 = min(n, a0 + step_rows)
                app_ms += timed_append(E[a0:a1])
                app_rows += a1 - a0
            del E
        row5 = ix5.store_view()[0].shape[1]
        fp8 = {"workload": f"C5: N={c5.N} (+{step_rows} rows appended before every batch size after the first) d={c5.d} "
                           f"fp8 e4m3 store with per-row scale, {c5.clusters}-cluster Zipf(1.1) mixture, k={c5.k}, "
                           "lambda=0, no mask; Q swept 1..8192",
               "append_rows_per_s": app_rows / (app_ms * 1e-3), "between_batches": [], "per_Q": {}}
        for Q in sweep:
            if Q != sweep[0]:                                     # the cache grows while it is being served
                E, U, M = wl5.rows(len(ix5), step_rows)
                ms_a = timed_append(E)
                fp8["between_batches"].append({"rows": step_rows, "ms": ms_a, "rows_per_s": step_rows / (ms_a * 1e-3),
                                               "GBps_in_plus_out": step_rows * (c5.d * 4 + row5 + 4) / (ms_a * 1e-3) / 1e9})
                del E
            n5 = len(ix5)
            bytes5 = n5 * (row5 + 4)   # rows + per-row scale
            qd = wl5.queries(Q, batch=Q)
            out_s = torch.empty(Q, c5.k, dtype=torch.float32, device=dev)
            out_i = torch.empty(Q, c5.k, dtype=torch.int64, device=dev)
            if Q >= 1024:
                st, wu = max(3, min(5, args.steps)), 1
            elif Q > 64:
                st, wu = max(3, min(10, args.steps)), 2
            else:
                st, wu = max(10, args.steps // 4), max(2, args.warmup // 4)
            ms, scan, wall, spread = time_search(ix5, torch, qd, c5.k, c5.lam, None, out_s, out_i, wu, st)
            flop = 2.0 * Q * n5 * c5.d
            rec = {"rows": n5, "queries_per_s": Q / (ms * 1e-3), "ms_per_step": ms, "steps": st, "scan_kernel_ms": scan,
                   "step_ms": spread, "scan_GBps": bytes5 / (scan * 1e-3) / 1e9,
                   "hbm_frac": bytes5 / (scan * 1e-3) / 1e9 / HBM_PEAK_GBS,
                   "scan_TFLOPs": flop / (scan * 1e-3) / 1e12,
                   "mfma_frac": flop / (scan * 1e-3) / 1e12 / MFMA_FP8_PEAK_TFLOPS,
                   "step_hbm_frac": bytes5 / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                   "step_mfma_frac": flop / (ms * 1e-3) / 1e12 / MFMA_FP8_PEAK_TFLOPS}
            if Q > 64:
                rec["tiles_again_blocks_redone"] = list(ix5.tiled_scan_counts())
            fp8["per_Q"][str(Q)] = rec
            del qd, out_s, out_i
            say(f"fp8 store Q={Q}: {ms:.2f} ms per step")
        ix5.close()

    say("fp8 store done")
    # ---- CPU reference on a bounded sample (rank 0, N = 1 only)
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ic_oracle
        qs = 64
        qh = wl.queries(64, batch=64)[:qs].cpu().numpy()
        t0 = time.perf_counter()
        scan = ic_oracle.Scan(qh, cfg.k, cfg.lam)      # the reference as it stands, fed chunk by chunk
        for part in sample_parts:
            scan.scan(part, None, None)
        scan.finish()
        dt = time.perf_counter() - t0
        n_sample = sum(p.shape[0] for p in sample_parts)
        full_equiv = qs / (dt * cfg.N / n_sample)
        cpu = {
            "value": full_equiv, "unit": "queries/s", "cores": ic_oracle.num_threads(), "kind": "oracle",
            "host": host_cpu(),
            "sample": f"{qs} queries x first {n_sample} rows in {dt:.2f} s, scaled linearly "
                      f"to N={cfg.N}",
        }

    achieved = headline["scan_GBps"]
    line = {
        "metric": "queries/sec for top-k example retrieval (N=10M, d=768)",
        "value": headline["queries_per_s"],
        "unit": "queries/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": headline["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"C3: N={cfg.N} d={cfg.d} bf16 store, {cfg.clusters}-cluster Zipf(1.1) mixture, "
                        f"k={cfg.k}, lambda=0, no mask; headline Q=64",
            "Q": 64, "k": cfg.k, "N": cfg.N, "d": cfg.d, "per_Q": per_q,
        },
        "append": {"rows_per_s": cfg.N / (append_ms * 1e-3),
                   "GBps_in_plus_out": cfg.N * (cfg.d * 4 + row_bytes + 4) / (append_ms * 1e-3) / 1e9},
        "roofline": {
            "bound": "hbm", "kernel": "scan_stream (similarity + fused partial top-k), Q=64",
            "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": SCAN_TRAFFIC_BYTES_Q64 if args.rows is None else None,
            "algorithmic_bytes_per_launch": store_bytes,
        },
        "cpu_baseline": cpu,
        "large_batch": large,
        "roofline_mfma": roof_mfma,
        "small_configs": small_cfgs,
        "fp8_store": fp8,
        "maintenance": maintenance,
        "census": census,
        "cluster_pruning": ivf_leg,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
