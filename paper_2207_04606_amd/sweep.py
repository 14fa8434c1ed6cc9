"""Parameter sweeps of the hyb(c,k) SpMM on one synthetic graph: the number of
column partitions c at a fixed feature size, and the feature size d at a fixed
c, each next to the single-pass CSR kernel ("no-hyb").  These are the two
ablations of Section 4.2.1 (speed-up against c with the cache hit rate, and
against d).  Run as

    python3 -m paper_2207_04606_amd.sweep [--config social] [--reps 20] [--only c|d]

Prints one line per point; every SpMM launch of a point can be matched to
profiler counters by its order (see --reps 1 for counter runs).
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="social")
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--only", choices=["c", "d"], default=None)
    ap.add_argument("--c-values", default="1,2,4,8,16")
    ap.add_argument("--d-values", default="32,64,128,256,512")
    ap.add_argument("--feat", type=int, default=128, help="feature size of the c sweep")
    args = ap.parse_args()

    import numpy as np
    import torch

    import paper_2207_04606_amd as sptir
    import workloads

    sptir.load_library()
    dev = torch.device("cuda:0")
    w = workloads.make_config(args.config)
    indptr = torch.from_numpy(w.indptr).to(dev)
    indices = torch.from_numpy(w.indices).to(dev)
    values = torch.from_numpy(w.values).to(dev)
    rng = np.random.Generator(np.random.PCG64(11))

    def timed(fn):
        for _ in range(2 if args.reps > 1 else 0):
            fn()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.reps

    def point(kind, c, feat, X, Y):
        # (through the search entry point with one candidate: its launch plan is sized for `feat`)
        hyb, _, _ = sptir.sptir_hyb_search(w.n_rows, w.n_cols, indptr, indices, values, feat, c_candidates=(c,),
                                           max_bucket_log2=w.max_bucket_log2, reps=1)
        info = sptir.sptir_hyb_info(hyb)
        ms = timed(lambda: sptir.sptir_spmm(hyb, X, Y))
        hyb.destroy()
        csr_ms = timed(lambda: sptir.sptir_spmm_csr(w.n_rows, w.n_cols, indptr, indices, values, X, Y))
        flops = 2.0 * w.nnz * feat
        print(json.dumps({"sweep": kind, "config": args.config, "c": c, "k": w.max_bucket_log2, "feat": feat,
                          "hyb_ms": round(ms, 4), "hyb_gflops": round(flops / ms / 1e6, 1),
                          "no_hyb_ms": round(csr_ms, 4), "no_hyb_gflops": round(flops / csr_ms / 1e6, 1),
                          "speedup": round(csr_ms / ms, 3), "launches": info["n_phases"],
                          "pad_pct_of_nnz": round(100.0 * info["n_pad_slots"] / max(info["nnz"], 1), 2),
                          "rem_nnz": info["n_rem_nnz"], "row_block": info["row_block"], "rounds": info["rounds"],
                          "heavy_pieces": info["n_heavy_pieces"]}), flush=True)

    if args.only in (None, "c"):
        X = torch.from_numpy(rng.standard_normal((w.n_cols, args.feat), dtype=np.float32)).to(dev)
        Y = torch.empty(w.n_rows, args.feat, device=dev)
        for c in [int(v) for v in args.c_values.split(",")]:
            point("c", c, args.feat, X, Y)
        del X, Y
    if args.only in (None, "d"):
        for feat in [int(v) for v in args.d_values.split(",")]:
            X = torch.from_numpy(rng.standard_normal((w.n_cols, feat), dtype=np.float32)).to(dev)
            Y = torch.empty(w.n_rows, feat, device=dev)
            point("d", w.n_col_parts, feat, X, Y)
            del X, Y


if __name__ == "__main__":
    main()
