#!/usr/bin/env python3
"""SpMM throughput of the hyb(c,k) path on one MI355X.

One "step" is one sptir_spmm call (Y = A X on the decomposed matrix, every
launch it enqueues) with A, X and Y resident in HBM.  The format conversion
(sptir_hyb_build) is pre-processing of a stationary matrix, as in the paper,
and is timed separately.  The workload is the largest graph of the benchmark
set (232,965 rows, ~114.6M non-zeros, hyb(16, 11)) at the metric's feature
size 128; the same graph at its as-written feature size 256 and the four
smaller configurations are reported in extra keys of the same JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published
GATHER_PEAK_GBS = 39300.0  # 256 CUs x 64 B/clk x 2.4 GHz vector-memory return path (measured ~38.7 TB/s)


def bytes_min(nnz, n_rows, n_cols, feat):
    """Minimal-traffic byte model: every true non-zero's column and value once, X once, Y once."""
    return 8.0 * nnz + 4.0 * n_cols * feat + 4.0 * n_rows * feat


def bytes_hyb(info, n_rows, n_cols, feat):
    """What the decomposition as stored has to move at the least: every ELL slot (pads included) and row id,
    every remainder non-zero and piece descriptor, X once, Y once."""
    return (8.0 * info["n_ell_slots"] + 4.0 * info["n_ell_rows"] + 8.0 * info["n_rem_nnz"] + 12.0 * info["n_rem_pieces"]
            + 4.0 * n_cols * feat + 4.0 * n_rows * feat)


def time_spmm(sptir, torch, hyb, X, Y, steps, warmup):
    for _ in range(warmup):
        sptir.sptir_spmm(hyb, X, Y)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        sptir.sptir_spmm(hyb, X, Y)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    event_ms = e0.elapsed_time(e1) / steps
    return wall_ms, event_ms


def time_graph_replay(sptir, torch, hyb, X, Y, calls_per_graph, replays):
    """sptir_spmm only enqueues kernels, so a stream capture records it: per-call time of replaying a graph of
    `calls_per_graph` calls (what a launch-bound small graph costs without the per-launch host work)."""
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for _ in range(calls_per_graph):
                sptir.sptir_spmm(hyb, X, Y, stream=side)
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(replays):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / (replays * calls_per_graph)


def time_cold(sptir, torch, hyb, X, Y, reps, scratch):
    """Per-step time with the caches flushed before every step (outside the timed region)."""
    times = []
    for _ in range(reps):
        scratch.add_(1.0)            # 1 GiB read + write: evicts L2 and the 256 MB Infinity Cache
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        sptir.sptir_spmm(hyb, X, Y)
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1))
    times.sort()
    return times[len(times) // 2]


def upload(torch, w):
    dev = torch.device("cuda:0")
    return (torch.from_numpy(w.indptr).to(dev), torch.from_numpy(w.indices).to(dev),
            torch.from_numpy(w.values).to(dev))


def read_traffic(key):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if one covers `key`."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == key:
            return float(parts[1])
    return None


def cpu_baseline(oracle, np, w, X_host, feat, budget_s=12.0):
    """The fp64 oracle, untuned, on a bounded sample of rows of the same workload."""
    rng = np.random.default_rng(1)
    rows = rng.permutation(w.n_rows).astype(np.int32)
    deg = np.diff(w.indptr)
    probe = rows[:2000]
    t0 = time.perf_counter()
    oracle.spmm_csr_rows(probe, w.indptr, w.indices, w.values, X_host)
    dt = max(time.perf_counter() - t0, 1e-4)
    rate = deg[probe].sum() / dt                       # non-zeros per second
    want_nnz = rate * budget_s
    csum = np.cumsum(deg[rows])
    n_sel = int(min(w.n_rows, max(2000, np.searchsorted(csum, want_nnz))))
    sel = rows[:n_sel]
    t0 = time.perf_counter()
    Yr, Sr = oracle.spmm_csr_rows(sel, w.indptr, w.indices, w.values, X_host)
    dt = time.perf_counter() - t0
    nnz_sel = int(deg[sel].sum())
    return dict(value=2.0 * nnz_sel * feat / dt / 1e9, unit="GFLOP/s", cores=oracle.num_threads(), kind="oracle",
                sample=f"{n_sel} random rows ({nnz_sel} non-zeros) of the same graph and X, feat={feat}, "
                       f"{dt:.1f} s, fp64, OpenMP over rows"), sel, Yr, Sr


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-extras", action="store_true", help="only the headline workload (for profiling runs)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (known HBM bytes) to scale profiler byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (every box has one); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2207_04606_amd as sptir
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    sptir.load_library()   # no fallback: raises if the HIP library is not built
    dev = torch.device("cuda:0")

    if args.copy_calibration:
        src = torch.ones(256 * 1024 * 1024, device=dev)   # 1 GiB written by the fill kernel
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)                      # 1 GiB read + 1 GiB written by one elementwise kernel
        torch.cuda.synchronize()
        del src, dst

    # ---------------------------------------------------------------- headline
    w = workloads.make_config("social")
    indptr, indices, values = upload(torch, w)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    hyb = sptir.sptir_hyb_build(w.n_rows, w.n_cols, indptr, indices, values, w.n_col_parts, w.max_bucket_log2)
    torch.cuda.synchronize()
    build_first_ms = (time.perf_counter() - t0) * 1e3
    t0 = time.perf_counter()
    hyb2 = sptir.sptir_hyb_build(w.n_rows, w.n_cols, indptr, indices, values, w.n_col_parts, w.max_bucket_log2)
    torch.cuda.synchronize()
    build_ms = (time.perf_counter() - t0) * 1e3
    hyb2.destroy()
    info = sptir.sptir_hyb_info(hyb)

    results = {}
    X_host_128 = None
    for feat in (128, 256):
        if feat == 256 and args.no_extras:
            continue
        if feat == w.feat:
            Xh = w.X
        else:
            Xh = np.random.Generator(np.random.PCG64(7)).standard_normal((w.n_cols, feat), dtype=np.float32)
        if feat == 128:
            X_host_128 = Xh
        X = torch.from_numpy(Xh).to(dev)
        Y = torch.empty(w.n_rows, feat, device=dev)
        wall_ms, event_ms = time_spmm(sptir, torch, hyb, X, Y, args.steps, args.warmup)
        flops = 2.0 * w.nnz * feat
        bmin = bytes_min(w.nnz, w.n_rows, w.n_cols, feat)
        results[feat] = dict(wall_ms=wall_ms, event_ms=event_ms, gflops=flops / wall_ms / 1e6,
                             bmin_gbs=bmin / event_ms / 1e6, bmin=bmin,
                             # one row of X (feat * 4 bytes) is gathered per non-zero; bucket pads are not walked
                             gather_gbs=w.nnz * feat * 4.0 / event_ms / 1e6,
                             Y=Y if feat == 128 else None)
        if feat == 256:
            del X, Y
    head = results[128]

    out = {
        "metric": "SpMM GFLOP/s and achieved HBM GB/s (% of peak) at feat=128, 1 MI355X",
        "value": round(head["gflops"], 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(head["wall_ms"], 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "largest graph of the set (social-like: 232,965 rows, %d non-zeros, power-law "
                               "degrees, values 1/deg) decomposed as hyb(c=16, k=11), X 232,965 x 128 fp32 N(0,1); "
                               "Y = A X per step" % w.nnz,
                   "n_rows": w.n_rows, "nnz": w.nnz, "feat": 128, "n_col_parts": w.n_col_parts,
                   "max_bucket_log2": w.max_bucket_log2, "stored_slots": info["n_ell_slots"] + info["n_rem_nnz"],
                   "pad_slots": info["n_pad_slots"], "walked_slots": info["n_work_items"] * info["item_slots"],
                   "kernel_launches_per_step": info["n_phases"],
                   "row_block": info["row_block"]},
        "hbm_gbs_min_model": round(head["bmin_gbs"], 1),
        "hbm_gbs_hyb_model": round(bytes_hyb(info, w.n_rows, w.n_cols, 128) / head["event_ms"] / 1e6, 1),
        "hbm_gbs_measured": None,
        "hbm_pct_of_peak": round(100.0 * head["bmin_gbs"] / HBM_PEAK_GBS, 2),
        "hyb_build_ms": round(build_ms, 3), "hyb_build_first_call_ms": round(build_first_ms, 3),
    }
    # dominant kernel: k_spmm_hyb, launched once per phase; events bracket all launches of a step
    per_launch_ms = head["event_ms"] / info["n_phases"]
    per_launch_bytes = head["bmin"] / info["n_phases"]
    out["roofline"] = {
        "bound": "hbm", "achieved": round(per_launch_bytes / per_launch_ms / 1e6, 1), "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(per_launch_bytes / per_launch_ms / 1e6 / HBM_PEAK_GBS, 4),
        "traffic": read_traffic("social_feat128"),
        "kernel": "k_spmm_hyb<4, 8, true, false>", "launches_per_step": info["n_phases"],
        "avg_launch_ms": round(per_launch_ms, 4), "algorithmic_bytes_per_launch": per_launch_bytes,
        # the path is a cache-served gather, not an HBM stream: each non-zero pulls feat*4 bytes of X
        # through the vector-memory return path, whose peak is 64 B/clk/CU
        "binding_roof": {"name": "vector-memory gather (L2 -> VGPR)", "achieved_gbs": round(head["gather_gbs"], 1),
                         "peak_gbs": GATHER_PEAK_GBS, "frac": round(head["gather_gbs"] / GATHER_PEAK_GBS, 4)},
    }

    if out["roofline"]["traffic"]:
        # bytes that crossed the L2 boundary per second (rocprofv3 counters of the committed profile run)
        out["hbm_gbs_measured"] = round(out["roofline"]["traffic"] / per_launch_ms / 1e6, 1)

    # ------------------------------------------------- CPU oracle beside it
    if not args.no_cpu:
        import oracle
        base, sel, Yr, Sr = cpu_baseline(oracle, np, w, X_host_128, 128)
        out["cpu_baseline"] = base
        Yg = head["Y"][torch.from_numpy(sel.astype(np.int64)).to(dev)].cpu().numpy().astype(np.float64)
        nz = Sr > 0
        out["max_normalised_error_vs_oracle"] = float((np.abs(Yg - Yr)[nz] / Sr[nz]).max())
    head["Y"] = None

    if not args.no_extras:
        r256 = results[256]
        out["as_written_feat256"] = {"gflops": round(r256["gflops"], 1), "ms_per_step": round(r256["wall_ms"], 4),
                                     "hbm_gbs_min_model": round(r256["bmin_gbs"], 1),
                                     "gather_gbs": round(r256["gather_gbs"], 1)}
        scratch = torch.zeros(256 * 1024 * 1024, device=dev)
        X = torch.from_numpy(X_host_128).to(dev)
        Y = torch.empty(w.n_rows, 128, device=dev)
        out["cold_ms_per_step"] = round(time_cold(sptir, torch, hyb, X, Y, 10, scratch), 4)
        # the single-pass CSR kernel ("no-hyb") on the same graph and X, for the comparison section 4.2.1 makes
        for _ in range(3):
            sptir.sptir_spmm_csr(w.n_rows, w.n_cols, indptr, indices, values, X, Y)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            sptir.sptir_spmm_csr(w.n_rows, w.n_cols, indptr, indices, values, X, Y)
        torch.cuda.synchronize()
        csr_ms = (time.perf_counter() - t0) * 1e3 / 10
        out["no_hyb_csr"] = {"ms_per_step": round(csr_ms, 4), "gflops": round(2.0 * w.nnz * 128 / csr_ms / 1e6, 1),
                             "hyb_speedup": round(csr_ms / head["wall_ms"], 3)}
        # the format search of section 4.2.1 (build every candidate c, time it, keep the fastest) over a few
        # partition counts around the configured one; the headline above stays at the configured c
        cands = [8, 12, 16, 24]
        t0 = time.perf_counter()
        best, best_c, cand_ms = sptir.sptir_hyb_search(w.n_rows, w.n_cols, indptr, indices, values, 128, cands,
                                                       w.max_bucket_log2, reps=5)
        torch.cuda.synchronize()
        search_ms = (time.perf_counter() - t0) * 1e3
        best_wall_ms, _ = time_spmm(sptir, torch, best, X, Y, 20, 3)
        best.destroy()
        out["format_search"] = {"candidates": cands, "ms_per_candidate": [round(m, 4) for m in cand_ms],
                                "best_c": best_c, "best_ms_per_step": round(best_wall_ms, 4),
                                "best_gflops": round(2.0 * w.nnz * 128 / best_wall_ms / 1e6, 1),
                                "search_ms": round(search_ms, 1)}
        # SDDMM on the same graph (B_ij = A_ij <X_i, Yt_j>), entries in CSR order and in column-partition order
        Xl = torch.randn(w.n_rows, 128, device=dev, generator=torch.Generator(device=dev).manual_seed(3))
        Bv = torch.empty(w.nnz, device=dev)

        def timed(fn, reps=10):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / reps

        sddmm_csr_ms = timed(lambda: sptir.sptir_sddmm_csr(w.n_rows, w.n_cols, indptr, indices, values, Xl, X, Bv))
        t0 = time.perf_counter()
        plan = sptir.sptir_sddmm_plan_build(w.n_rows, w.n_cols, indptr, indices, 0, 128)
        torch.cuda.synchronize()
        plan_ms = (time.perf_counter() - t0) * 1e3
        sddmm_ms = timed(lambda: sptir.sptir_sddmm(plan, values, Xl, X, Bv))
        pinfo = sptir.sptir_sddmm_plan_info(plan)
        plan.destroy()
        out["sddmm_feat128"] = {"ms_per_step": round(sddmm_ms, 4), "gflops": round(2.0 * w.nnz * 128 / sddmm_ms / 1e6, 1),
                                "n_col_parts": pinfo["n_col_parts"], "plan_build_ms": round(plan_ms, 3),
                                "gather_gbs": round(w.nnz * 512.0 / sddmm_ms / 1e6, 1),
                                "csr_order_ms_per_step": round(sddmm_csr_ms, 4)}
        del Xl, Bv
        # relational gather-matmul-scatter on a synthetic heterogeneous graph (51 relations, feature size 32)
        hw = workloads.make_hetero("hetero_d")
        hip_, hix, hva = (torch.from_numpy(a).to(dev) for a in (hw.indptr, hw.indices, hw.values))
        t0 = time.perf_counter()
        rg = sptir.sptir_rgms_build(hw.n_rel, hw.n, hw.n, hip_, hix, hva)
        torch.cuda.synchronize()
        rg_build_ms = (time.perf_counter() - t0) * 1e3
        rinfo = sptir.sptir_rgms_info(rg)
        hX, hW = torch.from_numpy(hw.X).to(dev), torch.from_numpy(hw.W).to(dev)
        hY = torch.empty(hw.n, 32, device=dev)
        rg_ms = timed(lambda: sptir.sptir_rgms(rg, hX, hW, hY), reps=20)
        pairs = rinfo["n_stacked_rows_stored"]
        out["rgms_feat32"] = {"workload": "%d nodes, %d relations, %d non-zeros, d_in = d_out = 32" % (hw.n, hw.n_rel, hw.nnz),
                              "ms_per_step": round(rg_ms, 4), "build_ms": round(rg_build_ms, 3),
                              "gflops": round((2.0 * hw.nnz * 32 + 2.0 * pairs * 32 * 32) / rg_ms / 1e6, 1),
                              "scatter_gbs": round(pairs * 128.0 / rg_ms / 1e6, 1), "tiles": rinfo["n_tiles"]}
        rg.destroy()
        del hX, hW, hY, hip_, hix, hva
        del X, Y
        hyb.destroy()
        del indptr, indices, values
        others = []
        for name in ("tiny", "small", "medium", "protein"):
            wc = workloads.make_config(name)
            ip, ix, va = upload(torch, wc)
            # (the first build at a new size loads kernels of the sort library: time the second)
            sptir.sptir_hyb_build(wc.n_rows, wc.n_cols, ip, ix, va, wc.n_col_parts, wc.max_bucket_log2).destroy()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            hc = sptir.sptir_hyb_build(wc.n_rows, wc.n_cols, ip, ix, va, wc.n_col_parts, wc.max_bucket_log2)
            torch.cuda.synchronize()
            b_ms = (time.perf_counter() - t0) * 1e3
            X = torch.from_numpy(wc.X).to(dev)
            Y = torch.empty(wc.n_rows, wc.feat, device=dev)
            wall_ms, event_ms = time_spmm(sptir, torch, hc, X, Y, 100, 10)
            cold = time_cold(sptir, torch, hc, X, Y, 10, scratch)
            bm = bytes_min(wc.nnz, wc.n_rows, wc.n_cols, wc.feat)
            others.append({"config": name, "nnz": wc.nnz, "feat": wc.feat,
                           "gflops": round(2.0 * wc.nnz * wc.feat / wall_ms / 1e6, 1),
                           "ms_per_step": round(wall_ms, 4),
                           "graph_replay_ms_per_step": round(time_graph_replay(sptir, torch, hc, X, Y, 10, 20), 4),
                           "cold_ms_per_step": round(cold, 4),
                           "hbm_gbs_min_model_cold": round(bm / cold / 1e6, 1), "hyb_build_ms": round(b_ms, 3)})
            hc.destroy()
        out["other_configs"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
