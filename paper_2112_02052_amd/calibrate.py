#!/usr/bin/env python3
"""Measures on this GPU where the per-window choice between the gather path and the MFMA tile path
should switch, and whether row clustering pays off on a given kind of graph.

    python -m paper_2112_02052_amd.calibrate [--sweep density|reuse|reorder|all] [--nodes N] [--features bf16|f32]

density  the paper's sparsity analysis (its table of dense blocks per row window): an N x N adjacency in
         which every 16-row window holds k fully dense 16 x 16 blocks, k = 1 .. 32, X bf16 N x 16; reports
         both paths in useful GFLOP/s (2 * nnz * D) and in the dense-equivalent GFLOP/s (2 * N * N * D)
         that the paper's numbers correspond to.  The paper uses N = 4096, where one call takes a few
         microseconds and measures the launch; the default here is 65,536 (pass --nodes 4096 for the
         paper's size).
reuse    windows with U distinct columns of which every row stores a fraction f, so the entries per
         distinct column (reuse = 16 f) sweep from 1 to 16: the tile path wins above the printed
         crossover, which is what the `min_reuse` argument of tcg_sgt_set_policy should be set to.
reorder  distinct columns per window and SpMM time before and after tcg_reorder_rows on the clustered
         and the R-MAT workloads.
Every line is also printed as JSON (prefix "JSON ") for scripts.
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--sweep", default="all", choices=["density", "reuse", "reorder", "all"])
    ap.add_argument("--nodes", type=int, default=65536)
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--features", default="bf16", choices=["bf16", "f32"],
                    help="feature type of the density and reuse sweeps (fp32 rows take the bf16-triple MFMA kernel)")
    args = ap.parse_args()

    import numpy as np
    import torch
    import paper_2112_02052_amd as tcg
    import workloads as W

    if not torch.cuda.is_available():
        print("calibrate needs a GPU", file=sys.stderr)
        sys.exit(2)
    tcg.load_library()
    dev = torch.device("cuda:0")

    def timed_us(fn):
        fn()
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(args.reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e3)
        return sorted(ts)[len(ts) // 2]

    feat_dtype = torch.bfloat16 if args.features == "bf16" else torch.float32

    def both_paths(g, D, dtype=feat_dtype):
        rp = torch.from_numpy(g.row_ptr).to(dev)
        ci = torch.from_numpy(g.col_idx).to(dev)
        meta = tcg.sgt_build(rp, ci, 16, 8, validate=False)
        X = torch.randn(g.n_cols, D, device=dev).to(dtype)
        Y = torch.empty(g.n_rows, D, device=dev)
        E = torch.empty(g.nnz, device=dev)
        res = {"U": meta.total_unique, "reuse": g.nnz / max(meta.total_unique, 1)}
        for name, pol in (("gather", tcg.POLICY_GATHER), ("tile", tcg.POLICY_TILE)):
            tcg.sgt_set_policy(meta, pol)
            res["spmm_%s_us" % name] = timed_us(lambda: tcg.spmm(meta, X, None, Y=Y))
            res["sddmm_%s_us" % name] = timed_us(lambda: tcg.sddmm(meta, X, out=E))
        meta.free()
        return res

    def emit(rec):
        print("JSON " + json.dumps(rec), flush=True)

    if args.sweep in ("density", "all"):
        n, D = args.nodes, 16
        print("density sweep: N = %d, D = %d, %s, k dense 16 x 16 blocks per window" % (n, D, args.features))
        print("  k  sparsity%%  nnz        spmm gather/tile us   useful GFLOP/s gather/tile   dense-equiv GFLOP/s gather/tile")
        for k in (1, 2, 4, 8, 16, 32):
            g = W.dense_block_windows(n, k, seed=1)
            r = both_paths(g, D)
            useful = [2.0 * g.nnz * D / r["spmm_%s_us" % p] / 1e3 for p in ("gather", "tile")]
            dense = [2.0 * n * n * D / r["spmm_%s_us" % p] / 1e3 for p in ("gather", "tile")]
            print("%3d  %8.2f  %9d  %9.1f /%8.1f   %12.0f /%8.0f   %16.0f /%10.0f" % (
                k, 100.0 * (1 - g.nnz / (n * n)), g.nnz, r["spmm_gather_us"], r["spmm_tile_us"], useful[0], useful[1],
                dense[0], dense[1]))
            emit(dict(sweep="density", n=n, D=D, features=args.features, blocks_per_window=k, nnz=g.nnz, **r))

    if args.sweep in ("reuse", "all"):
        n = args.nodes
        print("reuse sweep: N = %d, %s; entries per distinct column of a window = 16 * fill" % (n, args.features))
        print("  D    U_w  reuse   spmm gather/tile us    sddmm gather/tile us")
        for D in (32, 128, 256):
            for uw in (32, 128):
                cross = None
                prev = None
                for fill in (0.0625, 0.125, 0.1875, 0.25, 0.375, 0.5, 1.0):
                    g = W.window_fill(n, uw, fill, seed=2)
                    r = both_paths(g, D)
                    ratio = r["spmm_gather_us"] / r["spmm_tile_us"]
                    print("%4d  %4d  %5.2f  %9.1f /%8.1f    %9.1f /%8.1f" % (
                        D, uw, r["reuse"], r["spmm_gather_us"], r["spmm_tile_us"], r["sddmm_gather_us"], r["sddmm_tile_us"]))
                    emit(dict(sweep="reuse", n=n, D=D, features=args.features, unique_per_window=uw, fill=fill, **r))
                    if cross is None and ratio >= 1.0:
                        cross = r["reuse"] if prev is None else 0.5 * (prev + r["reuse"])
                    prev = r["reuse"]
                print("      -> SpMM tile path at least as fast from reuse ~ %s" % ("%.1f" % cross if cross else "never"))

    if args.sweep in ("reorder", "all"):
        print("row clustering: distinct columns per 16-row window and SpMM time, before / after (2 refinement rounds)")
        for name, cfg, kw in (("clustered, randomly relabelled", 5, {}), ("clustered, original order", 5, {"permute": False}),
                              ("R-MAT 100k", 3, {}), ("Chung-Lu 20k", 2, {})):
            c = W.make_config(cfg, **kw)
            g = c["csr"]
            rp = torch.from_numpy(g.row_ptr).to(dev)
            ci = torch.from_numpy(g.col_idx).to(dev)
            D = c["X"].shape[1]
            X = torch.randn(g.n_cols, D, device=dev).to(torch.bfloat16)
            Y = torch.empty(g.n_rows, D, device=dev)
            perm = tcg.reorder_rows(rp, ci, seed=0, refine=2)
            rp2, ci2, _ = tcg.csr_permute(rp, ci, perm, want_edge_perm=False)
            rec = dict(sweep="reorder", graph=name, nnz=g.nnz, D=D)
            for tag, (a, b) in (("before", (rp, ci)), ("after", (rp2, ci2))):
                meta = tcg.sgt_build(a, b, 16, 8, validate=False)
                rec["U_" + tag] = meta.total_unique
                rec["spmm_us_" + tag] = timed_us(lambda: tcg.spmm(meta, X, None, Y=Y))
                meta.free()
            print("  %-32s U %9d -> %9d   spmm bf16 D=%d  %8.1f -> %8.1f us" % (
                name, rec["U_before"], rec["U_after"], D, rec["spmm_us_before"], rec["spmm_us_after"]))
            emit(rec)


if __name__ == "__main__":
    main()
