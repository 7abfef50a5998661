#!/usr/bin/env python3
"""Times the three sparse kernels one by one on a square CSR matrix with power-law row lengths:
forward SpMM, transposed SpMM on the prebuilt mirror, and SDDMM.

    python -m paper_2407_17437_amd.kernel_bench [--n 16384] [--density 0.001 0.01 0.1] [--batch 128 1024]

Per case one JSON line: microseconds per launch (HIP events around `reps` back-to-back launches,
after a pass that evicts the caches), algorithmic GB/s and its fraction of the 8 TB/s HBM peak.
Algorithmic bytes: pattern and values once, dense operands once, result once; gathers that are
served by caches are not counted, so a fraction above what HBM could deliver means cache reuse.
`run_cases` is what bench.py calls for its table of the isolated kernels.
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


def kernel_bytes(kernel: str, n: int, nnz: int, batch: int) -> int:
    """Algorithmic bytes of one call on an n x n matrix (fp32 values, int32 indices)."""
    dense = 4 * batch * 2 * n                        # the dense operand in, the dense result out (SDDMM: both operands in)
    if kernel == "spmm_forward":
        return 8 * nnz + 4 * (n + 1) + dense + 4 * n
    if kernel == "spmm_transposed":                  # the stand-alone call refreshes the mirror's values first
        return 8 * nnz + 4 * (n + 1) + dense + 12 * nnz
    if kernel == "sddmm":                            # indices in, gradient out, bias gradient out
        return 8 * nnz + 4 * (n + 1) + dense + 4 * n
    raise KeyError(kernel)


def run_cases(n=16384, densities=(0.001, 0.01, 0.1), batches=(128, 1024), reps=20, uniform=False, partition="balanced",
              ld_pad=0, emit=None):
    """One record per (density, batch, kernel).  `partition`: balanced | row-split | prefer-staged
    (the latter two are measurement aids).  `ld_pad`: extra floats in the leading dimension of the dense matrices."""
    import numpy as np
    import torch
    from paper_2407_17437_amd import binding as nb
    from paper_2407_17437_amd import workloads as wl

    assert torch.cuda.is_available()
    mode = {"balanced": nb.NERVA_PARTITION_BALANCED, "row-split": nb.NERVA_PARTITION_ROW_SPLIT,
            "prefer-staged": nb.NERVA_PARTITION_PREFER_STAGED}[partition]
    nb.nerva_set_partition_mode(mode)
    flush = torch.empty(768 * 1024 * 1024 // 4, dtype=torch.float32, device="cuda")   # larger than every cache

    def timed(fn):
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

    out = []
    try:
        for dens in densities:
            if uniform:
                nnz = wl.round_half_up(dens * n * n)
                indptr, indices = wl.uniform_pattern(n, n, nnz, seed=11)
                lay = wl.SparseLayerData(n, n, indptr, indices, np.random.default_rng(12).standard_normal(nnz, dtype=np.float32),
                                         np.zeros(n, np.float32), False)
            else:
                lay = wl.make_zipf_matrix(n, dens, seed=11)
            rn = np.diff(lay.indptr)
            for batch in batches:
                L = nb.SparseLinear(lay, max_batch=batch)   # bound for this batch: the partition may depend on it
                rng = np.random.default_rng(batch)
                ld = nb.padded_ld(batch) + ld_pad
                X = nb.to_dense(rng.standard_normal((n, batch), dtype=np.float32), ld=ld)
                dY = nb.to_dense(rng.standard_normal((n, batch), dtype=np.float32), ld=ld)
                Y = nb.dense(n, batch, ld=ld); dX = nb.dense(n, batch, ld=ld)
                g = torch.empty(lay.nnz, device="cuda"); db = torch.empty(n, device="cuda")
                nnz = lay.nnz
                cases = {
                    "spmm_forward": lambda: nb.sparse_linear_forward(L.handle, X, Y, batch),
                    "spmm_transposed": lambda: nb.sparse_linear_backward(L.handle, None, None, dY, dX, None, None, batch),
                    "sddmm": lambda: nb.sparse_linear_backward(L.handle, X, None, dY, None, g, db, batch),
                }
                for name, fn in cases.items():
                    byt = kernel_bytes(name, n, nnz, batch)
                    cold, warm = timed(fn)
                    rec = {
                        "kernel": name, "n": n, "density": dens, "nnz": nnz, "batch": batch,
                        "rows": "uniform" if uniform else "zipf1.2", "partition": partition,
                        "max_row": int(rn.max()), "median_row": float(np.median(rn)),
                        "us_cold": round(cold, 2), "us_back_to_back": round(warm, 2), "algorithmic_MB": round(byt / 1e6, 2),
                        "gflop": round(2.0 * nnz * batch / 1e9, 3),
                        "gbs_cold": round(byt / cold / 1e3, 1), "frac_hbm_cold": round(byt / cold / 1e3 / HBM_PEAK_GBS, 4),
                        "gbs_back_to_back": round(byt / warm / 1e3, 1),
                        "frac_hbm_back_to_back": round(byt / warm / 1e3 / HBM_PEAK_GBS, 4),
                        "tflops_back_to_back": round(2.0 * nnz * batch / warm / 1e6, 3)}
                    if ld_pad:
                        rec["ld"] = ld
                    out.append(rec)
                    if emit:
                        emit(rec)
                L.close()
                del X, dY, Y, dX, g, db
    finally:
        nb.nerva_set_partition_mode(nb.NERVA_PARTITION_BALANCED)
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=16384)
    ap.add_argument("--density", type=float, nargs="+", default=[0.001, 0.01, 0.1])
    ap.add_argument("--batch", type=int, nargs="+", default=[128, 1024])
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--uniform", action="store_true", help="uniform random pattern instead of power-law rows")
    ap.add_argument("--ld-pad", type=int, default=0, help="extra floats in the leading dimension of the dense matrices")
    ap.add_argument("--prefer-staged", action="store_true",
                    help="measurement aid: staged (LDS) kernels wherever they can run, not only where the library expects them to pay")
    ap.add_argument("--row-split", action="store_true",
                    help="build the layers with plain row splitting (one wave per row) instead of the balanced partition")
    args = ap.parse_args()
    partition = "row-split" if args.row_split else ("prefer-staged" if args.prefer_staged else "balanced")
    run_cases(args.n, args.density, args.batch, args.reps, args.uniform, partition, args.ld_pad,
              emit=lambda rec: print(json.dumps(rec), flush=True))
    return 0


if __name__ == "__main__":
    sys.exit(main())
