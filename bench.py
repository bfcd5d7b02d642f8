#!/usr/bin/env python3
"""Benchmark of the neighbour-aggregation hot path on one MI355X.

Workload: the large-SpMM configuration (1,000,000-node R-MAT graph, ~10M sampled pairs
deduplicated and symmetrised, unit edge values, X fp32 1M x 128, fp32 accumulation, Y fp32),
synthetic and seeded.  One step = one pass of the whole path on inputs resident in HBM:
    tcg_sgt_build (graph translation) -> tcg_spmm (neighbour aggregation) -> tcg_sddmm (edge features)
Each part is bracketed by HIP events on the stream the library launches on.

The printed JSON line reports
  value              useful SpMM GFLOP/s = 2 * nnz * D / (mean tcg_spmm time of the timed steps)
  ms_per_step        wall time of one whole step (translation + SpMM + SDDMM)
  roofline           algorithmic SpMM bytes per call / mean tcg_spmm time, against 8 TB/s HBM
  cpu_baseline       the CPU oracle's SpMM timed on the host cores, same inputs
plus the SDDMM edge rate, the bf16-feature SpMM numbers and the translation time.
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


def algorithmic_bytes_spmm(n_rows, nnz, U, n_win, D, s_x, s_y, weighted):
    """Bytes the method itself has to move for one SpMM: every window-unique neighbour row of X
    once, Y once, the translated-graph indices once."""
    return (U * D * s_x + n_rows * D * s_y + 4 * U + 4 * nnz + (4 * nnz if weighted else 0)
            + 4 * (n_rows + 1) + 8 * (n_win + 1))


def algorithmic_bytes_sddmm(n_rows, nnz, U, n_win, D, s_x):
    return U * D * s_x + n_rows * D * s_x + 4 * nnz + 4 * U + 4 * nnz + 4 * (n_rows + 1) + 8 * (n_win + 1)


def read_traffic():
    """HBM bytes per tcg_spmm call measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE runs),
    as summarised under profiles/; None when no summary is present."""
    path = os.path.join(ROOT, "profiles", "spmm_rmat1m_d128_f32_hbm_traffic.json")
    try:
        with open(path) as f:
            return float(json.load(f)["hbm_bytes_per_spmm_call"])
    except Exception:
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--nodes", type=int, default=1000000, help="node count of the R-MAT workload")
    ap.add_argument("--dim", type=int, default=128)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 512 MiB device copy (reference dispatch for HBM counter scaling)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2112_02052_amd as tcg
    import workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    tcg.load_library()
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    t0 = time.time()
    c = W.make_config(4, n=args.nodes, d=args.dim)
    g, X = c["csr"], c["X"]
    N, nnz, D = g.n_rows, g.nnz, args.dim
    gen_s = time.time() - t0
    rp = torch.from_numpy(g.row_ptr).to(dev)
    ci = torch.from_numpy(g.col_idx).to(dev)
    Xf = torch.from_numpy(X).to(dev)
    Xb = torch.from_numpy(W.round_to_bf16(X)).to(dev).to(torch.bfloat16)
    Y = torch.empty((N, D), dtype=torch.float32, device=dev)
    E = torch.empty(nnz, dtype=torch.float32, device=dev)
    H, TW = 16, 8

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def one_step(record):
        e = [ev() for _ in range(4)]
        e[0].record()
        meta = tcg.sgt_build(rp, ci, H, TW, validate=False)
        e[1].record()
        tcg.spmm(meta, Xf, None, Y=Y)
        e[2].record()
        tcg.sddmm(meta, Xf, out=E)
        e[3].record()
        if record is not None:
            record.append(e)
        return meta

    meta = None
    for _ in range(args.warmup):
        if meta is not None:
            meta.free()
        meta = one_step(None)
    torch.cuda.synchronize()
    events = []
    t_start = time.perf_counter()
    for _ in range(args.steps):
        if meta is not None:
            meta.free()
        meta = one_step(events)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    ms_per_step = wall * 1e3 / args.steps
    sgt_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in events]))
    spmm_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in events]))
    sddmm_ms = float(np.mean([e[2].elapsed_time(e[3]) for e in events]))

    U, n_win, tiles = meta.total_unique, meta.n_windows, meta.total_tiles
    plan = tcg.sgt_plan_stats(meta)

    # Steady state of the two kernels with the translated graph reused (how training uses it).
    def timed_loop(fn, reps):
        fn()
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    reps = max(5, args.steps)
    spmm_f32_loop_ms = timed_loop(lambda: tcg.spmm(meta, Xf, None, Y=Y), reps)
    spmm_bf16_loop_ms = timed_loop(lambda: tcg.spmm(meta, Xb, None, Y=Y), reps)
    sddmm_f32_loop_ms = timed_loop(lambda: tcg.sddmm(meta, Xf, out=E), reps)
    sddmm_bf16_loop_ms = timed_loop(lambda: tcg.sddmm(meta, Xb, out=E), reps)

    b_f32 = algorithmic_bytes_spmm(N, nnz, U, n_win, D, 4, 4, False)
    b_bf16 = algorithmic_bytes_spmm(N, nnz, U, n_win, D, 2, 4, False)
    b_sddmm = algorithmic_bytes_sddmm(N, nnz, U, n_win, D, 4)
    flops = 2.0 * nnz * D
    achieved = b_f32 / (spmm_ms * 1e-3) / 1e9

    out = {
        "metric": "SpMM useful GFLOP/s + HBM GB/s (1M nodes, D=128); SDDMM Gedges/s",
        "value": flops / (spmm_ms * 1e-3) / 1e9,
        "unit": "GFLOP/s (useful, SpMM)",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "config 4: R-MAT N=%d, %d stored entries, unit edge values, X fp32 N x %d, "
                               "window 16 x 8; step = sgt_build + spmm + sddmm" % (N, nnz, D),
                   "nnz": nnz, "window_unique_total": U, "tiles": tiles, "windows": n_win,
                   "tile_windows": plan["n_tile_windows"], "segments": plan["n_segments"],
                   "long_rows": plan["n_long_rows"]},
        "step_parts_ms": {"sgt_build": sgt_ms, "spmm": spmm_ms, "sddmm": sddmm_ms},
        "spmm_hbm_gbs_algorithmic": achieved,
        "sddmm_gedges_per_s": nnz / (sddmm_ms * 1e-3) / 1e9,
        "sddmm_hbm_gbs_algorithmic": b_sddmm / (sddmm_ms * 1e-3) / 1e9,
        "sgt_medges_per_s": nnz / (sgt_ms * 1e-3) / 1e6,
        "steady_state": {
            "spmm_f32_ms": spmm_f32_loop_ms, "spmm_f32_gflops": flops / spmm_f32_loop_ms / 1e6,
            "spmm_f32_frac_hbm": b_f32 / (spmm_f32_loop_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "spmm_bf16_ms": spmm_bf16_loop_ms, "spmm_bf16_gflops": flops / spmm_bf16_loop_ms / 1e6,
            "spmm_bf16_frac_hbm": b_bf16 / (spmm_bf16_loop_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "sddmm_f32_ms": sddmm_f32_loop_ms, "sddmm_f32_gedges": nnz / sddmm_f32_loop_ms / 1e6,
            "sddmm_bf16_ms": sddmm_bf16_loop_ms, "sddmm_bf16_gedges": nnz / sddmm_bf16_loop_ms / 1e6,
        },
        "roofline": {"bound": "hbm", "kernel": "tcg_spmm (spmm_gather_kernel + spmm_reduce_long_kernel)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": read_traffic(),
                     "algorithmic_bytes": b_f32},
        "generate_s": gen_s,
    }

    if not args.no_cpu_baseline:
        import oracle
        oracle.spmm(g.row_ptr, g.col_idx, X)                      # warm-up
        ts = []
        for _ in range(9):
            t1 = time.perf_counter()
            oracle.spmm(g.row_ptr, g.col_idx, X)
            ts.append(time.perf_counter() - t1)
        t_cpu = sorted(ts)[len(ts) // 2]
        out["cpu_baseline"] = {"value": flops / t_cpu / 1e9, "unit": "GFLOP/s (useful, SpMM)",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "the full workload (all %d rows), fp64-accumulate CSR SpMM, median of 9 runs, "
                                         "%.2f s each" % (N, t_cpu)}
    if args.calibrate_copy:
        src = torch.empty(128 << 20, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                                            # reads 512 MiB, writes 512 MiB
        torch.cuda.synchronize()
    meta.free()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
