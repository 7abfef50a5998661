#!/usr/bin/env python3
"""Times the three sparse kernels one by one on a square CSR matrix with power-law row lengths:
forward SpMM, transposed SpMM on the prebuilt mirror, and SDDMM.

    python -m paper_2407_17437_amd.kernel_bench [--n 16384] [--density 0.001 0.01 0.1] [--batch 128 1024]

Per case one JSON line: microseconds per launch (HIP events around `reps` back-to-back launches,
after a pass that evicts the caches), algorithmic GB/s and its fraction of the 8 TB/s HBM peak.
Algorithmic bytes: pattern and values once, dense operands once, result once; gathers that are
served by caches are not counted, so a fraction above what HBM could deliver means cache reuse.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=16384)
    ap.add_argument("--density", type=float, nargs="+", default=[0.001, 0.01, 0.1])
    ap.add_argument("--batch", type=int, nargs="+", default=[128, 1024])
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--uniform", action="store_true", help="uniform random pattern instead of power-law rows")
    ap.add_argument("--prefer-staged", action="store_true",
                    help="measurement aid: staged (LDS) kernels wherever they can run, not only where the library expects them to pay")
    ap.add_argument("--row-split", action="store_true",
                    help="build the layers with plain row splitting (one wave per row) instead of the balanced partition")
    args = ap.parse_args()

    import numpy as np
    import torch
    from paper_2407_17437_amd import binding as nb
    from paper_2407_17437_amd import workloads as wl

    assert torch.cuda.is_available()
    if args.row_split:
        nb.nerva_set_partition_mode(nb.NERVA_PARTITION_ROW_SPLIT)
    if args.prefer_staged:
        nb.nerva_set_partition_mode(nb.NERVA_PARTITION_PREFER_STAGED)
    n = args.n
    flush = torch.empty(768 * 1024 * 1024 // 4, dtype=torch.float32, device="cuda")   # larger than every cache

    def timed(fn, reps):
        fn()                                            # warm-up: code objects, first touch
        times = []
        for _ in range(reps):
            flush.add_(1.0)                             # evict L2 / infinity cache
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); fn(); e1.record()
            e1.synchronize()
            times.append(e0.elapsed_time(e1) * 1e3)
        cold = float(np.median(times))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record(); e1.synchronize()
        return cold, e0.elapsed_time(e1) * 1e3 / reps

    for dens in args.density:
        if args.uniform:
            nnz = wl.round_half_up(dens * n * n)
            indptr, indices = wl.uniform_pattern(n, n, nnz, seed=11)
            lay = wl.SparseLayerData(n, n, indptr, indices, np.random.default_rng(12).standard_normal(nnz, dtype=np.float32),
                                     np.zeros(n, np.float32), False)
        else:
            lay = wl.make_zipf_matrix(n, dens, seed=11)
        rn = np.diff(lay.indptr)
        for batch in args.batch:
            L = nb.SparseLinear(lay, max_batch=batch)   # bound for this batch: the partition may depend on it
            rng = np.random.default_rng(batch)
            X = nb.to_dense(rng.standard_normal((n, batch), dtype=np.float32))
            dY = nb.to_dense(rng.standard_normal((n, batch), dtype=np.float32))
            Y = nb.dense(n, batch); dX = nb.dense(n, batch)
            g = torch.empty(lay.nnz, device="cuda"); db = torch.empty(n, device="cuda")
            nnz = lay.nnz
            cases = {
                "spmm_forward": (lambda: nb.sparse_linear_forward(L.handle, X, Y, batch),
                                 8 * nnz + 4 * (n + 1) + 4 * batch * 2 * n + 4 * n),
                "spmm_transposed": (lambda: nb.sparse_linear_backward(L.handle, None, None, dY, dX, None, None, batch),
                                    8 * nnz + 4 * (n + 1) + 4 * batch * 2 * n + 12 * nnz),   # + mirror value refresh
                "sddmm": (lambda: nb.sparse_linear_backward(L.handle, X, None, dY, None, g, db, batch),
                          8 * nnz + 4 * (n + 1) + 4 * batch * 2 * n + 4 * n),
            }
            for name, (fn, byt) in cases.items():
                cold, warm = timed(fn, args.reps)
                print(json.dumps({
                    "kernel": name, "n": n, "density": dens, "nnz": nnz, "batch": batch,
                    "rows": "uniform" if args.uniform else "zipf1.2",
                    "partition": "row-split" if args.row_split else ("prefer-staged" if args.prefer_staged else "balanced"), "max_row": int(rn.max()), "median_row": float(np.median(rn)),
                    "us_cold": round(cold, 2), "us_back_to_back": round(warm, 2), "algorithmic_MB": round(byt / 1e6, 2),
                    "gflop": round(2.0 * nnz * batch / 1e9, 3),
                    "gbs_cold": round(byt / cold / 1e3, 1), "frac_hbm_cold": round(byt / cold / 1e3 / HBM_PEAK_GBS, 4),
                    "gbs_back_to_back": round(byt / warm / 1e3, 1),
                    "tflops_back_to_back": round(2.0 * nnz * batch / warm / 1e6, 3)}), flush=True)
            L.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
