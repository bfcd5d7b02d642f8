#!/usr/bin/env python3
"""Benchmark of the neighbour-aggregation hot path on one MI355X.

Headline workload ("4"): the large-SpMM configuration -- 1,000,000-node R-MAT graph (~10M sampled pairs,
deduplicated and symmetrised), unit edge values, X fp32 1M x 128, fp32 accumulation, Y fp32; synthetic
and seeded.  One step = one pass of the whole path on inputs resident in HBM:
    tcg_sgt_build (graph translation) -> tcg_spmm (neighbour aggregation) -> tcg_sddmm (edge features)
Each part is bracketed by HIP events on the stream the library launches on.

The printed JSON line reports
  value              useful SpMM GFLOP/s = 2 * nnz * D / (median tcg_spmm time of the timed steps)
  ms_per_step        wall time of one whole step
  roofline           the SpMM launch priced three ways against 8 TB/s: `frac` with the method's algorithmic
                     bytes (every window-unique neighbour row once -- caches can serve more than that, so it
                     is not bounded by 1), `frac_counter` with the HBM-side bytes that rocprofv3 counted for
                     the same kernels (from profiles/, dropped when the kernel sources changed since), and
                     `frac_compulsory` with every X row once
  cpu_baseline       the CPU oracle's SpMM timed on the host cores, same inputs (plus the float-accumulating
                     variants and the window-parallel translation, each with its core count)
  d_sweep            SpMM / SDDMM on the headline graph for feature widths 16 .. 256 in both feature types (the
                     paper's embedding-dimension study, section 5.4)
  configs            with no --workload: a few steps of every other workload x feature type (ms as median
                     and minimum, GFLOP/s, Gedges/s, byte counts, tile share, tile counts with and without the
                     translation, largest normalised error against the oracle on the full outputs)

--workload selects one workload (1, 2, 3, 4, 5, or 5a = workload 5 without the random relabelling, the case
where windows share neighbours and the MFMA tile path is chosen) as the headline and skips `configs`; its
steps run the operations that workload lists (3: SDDMM -> row softmax -> SpMM).  --features overrides the
feature type (f32 / bf16).
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
METRIC = "SpMM useful GFLOP/s + HBM GB/s (1M nodes, D=128); SDDMM Gedges/s"

WORKLOADS = {
    # name: (config number, permute, default feature type, operations after the translation)
    "1": (1, True, "f32", ("spmm",)),
    "2": (2, True, "f32", ("spmm",)),
    "3": (3, True, "f32", ("sddmm", "row_softmax", "spmm_w")),
    "4": (4, True, "f32", ("spmm", "sddmm")),
    "5": (5, True, "bf16", ("sddmm", "spmm")),
    "5a": (5, False, "bf16", ("sddmm", "spmm")),
}
# (workload, feature type, row-clustering rounds) run after the headline when no --workload is given
OTHER_CONFIGS = [("4", "bf16", None), ("1", "f32", None), ("2", "f32", None), ("3", "f32", None),
                 ("5", "bf16", None), ("5", "bf16", 2), ("5a", "bf16", None), ("5a", "f32", None)]
# sources whose change invalidates a stored counter measurement of the SpMM kernels
TRAFFIC_SOURCES = ["paper_2112_02052_amd/csrc/spmm.hip", "paper_2112_02052_amd/csrc/spmm_tile.hip",
                   "paper_2112_02052_amd/csrc/sgt.hip", "paper_2112_02052_amd/csrc/common.h",
                   "paper_2112_02052_amd/csrc/devutil.h"]
SX = {"f32": 4, "bf16": 2}


def algorithmic_bytes_spmm(n_rows, nnz, U, n_win, D, s_x, s_y, weighted):
    """Bytes the method itself has to move for one SpMM: every window-unique neighbour row of X
    once, Y once, the translated-graph indices once."""
    return (U * D * s_x + n_rows * D * s_y + 4 * U + 4 * nnz + (4 * nnz if weighted else 0)
            + 4 * (n_rows + 1) + 8 * (n_win + 1))


def algorithmic_bytes_sddmm(n_rows, nnz, U, n_win, D, s_x):
    return U * D * s_x + n_rows * D * s_x + 4 * nnz + 4 * U + 4 * nnz + 4 * (n_rows + 1) + 8 * (n_win + 1)


def source_hashes():
    out = {}
    for rel in TRAFFIC_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            out[rel] = hashlib.sha256(f.read()).hexdigest()[:16]
    return out


def read_traffic(workload, features):
    """HBM-side bytes per tcg_spmm call counted by rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE runs), as
    summarised under profiles/.  Returns (bytes, record) or (None, reason): the summary names the kernel
    sources it was measured with, and a figure whose sources have changed since is not reported."""
    name = {("4", "f32"): "spmm_rmat1m_d128_f32_hbm_traffic.json",
            ("4", "bf16"): "spmm_rmat1m_d128_bf16_hbm_traffic.json",
            ("5a", "bf16"): "spmm_clustered5a_d256_bf16_hbm_traffic.json"}.get((workload, features))
    if name is None:
        return None, "no counter summary for this workload"
    try:
        with open(os.path.join(ROOT, "profiles", name)) as f:
            rec = json.load(f)
    except Exception:
        return None, "no counter summary for this workload"
    if rec.get("sources") != source_hashes():
        return None, "kernel sources changed since profiles/%s was measured" % name
    return float(rec["hbm_bytes_per_spmm_call"]), {"file": "profiles/" + name, "kernels": rec.get("kernels")}


def stats(values):
    import numpy as np
    v = np.asarray(values, dtype=np.float64)
    return {"median": float(np.median(v)), "min": float(v.min()), "mean": float(v.mean()), "n": int(v.size)}


def norm_err(got, ref):
    import numpy as np
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-300))


class Run:
    """One workload on the GPU: inputs uploaded once, then timed steps and steady-state loops."""

    def __init__(self, workload, feat, args, reorder=None):
        import torch
        import paper_2112_02052_amd as tcg
        import workloads as W
        self.torch, self.tcg, self.W = torch, tcg, W
        self.workload, self.args = workload, args
        cfg, permute, default_feat, self.ops = WORKLOADS[workload]
        self.feat = feat or default_feat
        dev = torch.device("cuda:0")
        t0 = time.time()
        self.c = c = W.make_config(cfg, n=args.nodes, d=args.dim, permute=permute, x_dtype=self.feat)
        self.gen_s = time.time() - t0
        self.g, self.X = c["csr"], c["X"]
        g = self.g
        self.N, self.nnz, self.D = g.n_rows, g.nnz, self.X.shape[1]
        tdt = {"f32": torch.float32, "bf16": torch.bfloat16}
        self.rp = torch.from_numpy(g.row_ptr).to(dev)
        self.ci = torch.from_numpy(g.col_idx).to(dev)
        self.Xd = {self.feat: torch.from_numpy(self.X).to(dev).to(tdt[self.feat])}
        other = "bf16" if self.feat == "f32" else "f32"
        self.Xd[other] = (torch.from_numpy(W.round_to_bf16(self.X)).to(dev).to(torch.bfloat16) if other == "bf16"
                          else torch.from_numpy(self.X).to(dev))
        self.w_given = torch.from_numpy(c["w"]).to(dev) if c["w"] is not None else None
        self.H, self.TW = args.window_height, 8
        self.reorder_info = None
        self.perm = None
        if reorder is not None:
            self._cluster(reorder)
        self.Y = torch.empty((self.N, self.D), dtype=torch.float32, device=dev)
        self.E = torch.empty(self.nnz, dtype=torch.float32, device=dev)
        self.P = torch.empty(self.nnz, dtype=torch.float32, device=dev)
        self.weighted = self.w_given is not None or "spmm_w" in self.ops
        self.spmm_op = "spmm_w" if "spmm_w" in self.ops else "spmm"
        self.meta = None

    def _cluster(self, rounds):
        torch, tcg = self.torch, self.tcg

        def once_ms(fn):
            torch.cuda.synchronize()
            t = time.perf_counter()
            r = fn()
            torch.cuda.synchronize()
            return r, (time.perf_counter() - t) * 1e3
        rp, ci = self.rp, self.ci
        tcg.reorder_rows(rp, ci, seed=0, refine=rounds)                  # warm-up (fills the allocator cache)
        perm, t_perm = once_ms(lambda: tcg.reorder_rows(rp, ci, seed=0, refine=rounds))
        tcg.csr_permute(rp, ci, perm)
        (rp2, ci2, ep), t_csr = once_ms(lambda: tcg.csr_permute(rp, ci, perm))
        pl = perm.long()
        _, t_x = once_ms(lambda: self.Xd[self.feat][pl])
        u_before = tcg.sgt_build(rp, ci, self.H, self.TW, validate=False)
        # the same three steps as one library call (clustering + relabelling + translation)
        (m1, _, _), t_one = once_ms(lambda: tcg.sgt_build_clustered(rp, ci, self.H, self.TW, seed=0, refine=rounds))
        m1.free()
        self.reorder_info = {"refine_rounds": rounds, "reorder_rows_ms": t_perm, "csr_permute_ms": t_csr,
                             "permute_X_ms": t_x, "sgt_build_clustered_ms": t_one,
                             "window_unique_before": u_before.total_unique}
        u_before.free()
        self.rp, self.ci, self.perm = rp2, ci2, perm
        self.Xd = {k: v[pl].contiguous() for k, v in self.Xd.items()}
        if self.w_given is not None:
            self.w_given = tcg.edge_gather(ep, self.w_given)

    def ev(self):
        return self.torch.cuda.Event(enable_timing=True)

    def run_op(self, op, x):
        tcg, meta = self.tcg, self.meta
        if op == "spmm":
            tcg.spmm(meta, x, self.w_given, Y=self.Y)
        elif op == "spmm_w":
            tcg.spmm(meta, x, self.P, Y=self.Y)
        elif op == "sddmm":
            tcg.sddmm(meta, x, out=self.E)
        elif op == "row_softmax":
            tcg.row_softmax(meta, self.E, out=self.P)

    def one_step(self, record):
        e = [self.ev() for _ in range(len(self.ops) + 2)]
        e[0].record()
        self.meta = self.tcg.sgt_build(self.rp, self.ci, self.H, self.TW, validate=False)
        e[1].record()
        for k, op in enumerate(self.ops):
            self.run_op(op, self.Xd[self.feat])
            e[k + 2].record()
        if record is not None:
            record.append(e)

    def steps(self, steps, warmup):
        """W untimed steps, then exactly K timed ones.  Returns (wall ms per step, {part: stats})."""
        torch = self.torch
        for _ in range(warmup):
            if self.meta is not None:
                self.meta.free()
            self.one_step(None)
        torch.cuda.synchronize()
        events = []
        t_start = time.perf_counter()
        for _ in range(steps):
            if self.meta is not None:
                self.meta.free()
            self.one_step(events)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t_start
        parts = {"whole_step_gpu": stats([e[0].elapsed_time(e[-1]) for e in events]),
                 "sgt_build": stats([e[0].elapsed_time(e[1]) for e in events])}
        for k, op in enumerate(self.ops):
            parts[op.replace("spmm_w", "spmm")] = stats([e[k + 1].elapsed_time(e[k + 2]) for e in events])
        return wall * 1e3 / steps, parts

    def timed(self, fn, reps):
        """Per-call HIP event timing of `reps` calls after one warm-up call: median / min / mean in ms."""
        torch = self.torch
        fn()
        torch.cuda.synchronize()
        pairs = []
        for _ in range(reps):
            a, b = self.ev(), self.ev()
            a.record()
            fn()
            b.record()
            pairs.append((a, b))
        torch.cuda.synchronize()
        return stats([a.elapsed_time(b) for a, b in pairs])

    def timed_loop(self, fn, reps):
        """Mean time of `reps` calls issued back to back between one pair of events (launch cost overlapped)."""
        torch = self.torch
        fn()
        torch.cuda.synchronize()
        a, b = self.ev(), self.ev()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    def sizes(self):
        meta = self.meta
        plan = self.tcg.sgt_plan_stats(meta)
        t8, u8 = self.tcg.sgt_tile_stats(meta, 8)
        t16, u16 = self.tcg.sgt_tile_stats(meta, 16)
        tile_share = plan["nnz_tile"] / max(self.nnz, 1)
        return {"nnz": self.nnz, "window_unique_total": meta.total_unique, "windows": meta.n_windows,
                "tile_windows": plan["n_tile_windows"], "tile_edge_share": tile_share,
                "segments": plan["n_segments"], "long_rows": plan["n_long_rows"],
                # the paper's SGT-effectiveness quantity (section 5.2): tiles a tiled kernel visits
                "tiles_w8": {"translated": t8, "untranslated": u8, "reduction": 1.0 - t8 / max(u8, 1)},
                "tiles_w16": {"translated": t16, "untranslated": u16, "reduction": 1.0 - t16 / max(u16, 1)}}

    def byte_counts(self, feat):
        N, nnz, D, meta = self.N, self.nnz, self.D, self.meta
        U, n_win = meta.total_unique, meta.n_windows
        b_alg = algorithmic_bytes_spmm(N, nnz, U, n_win, D, SX[feat], 4, self.weighted)
        return {"spmm_algorithmic": b_alg,
                # brackets: every X row once (a lower bound for any method) / once per stored entry (no reuse)
                "spmm_compulsory": b_alg - U * D * SX[feat] + self.g.n_cols * D * SX[feat],
                "spmm_csr_gather": algorithmic_bytes_spmm(N, nnz, nnz, n_win, D, SX[feat], 4, self.weighted),
                "sddmm_algorithmic": algorithmic_bytes_sddmm(N, nnz, U, n_win, D, SX[feat])}

    def steady(self, reps, feats):
        """Kernels on a reused translated graph (how training uses it), per feature type."""
        out = {}
        flops = 2.0 * self.nnz * self.D
        for f in feats:
            b = self.byte_counts(f)
            sp = self.timed(lambda: self.run_op(self.spmm_op, self.Xd[f]), reps)
            sd = self.timed(lambda: self.run_op("sddmm", self.Xd[f]), reps)
            out[f] = {"spmm_ms": sp, "spmm_gflops": flops / sp["median"] / 1e6,
                      "spmm_frac_hbm_algorithmic": b["spmm_algorithmic"] / (sp["median"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      "spmm_loop_ms": self.timed_loop(lambda: self.run_op(self.spmm_op, self.Xd[f]), reps),
                      "sddmm_ms": sd, "sddmm_gedges": self.nnz / sd["median"] / 1e6,
                      "sddmm_frac_hbm_algorithmic": b["sddmm_algorithmic"] / (sd["median"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      "sddmm_loop_ms": self.timed_loop(lambda: self.run_op("sddmm", self.Xd[f]), reps)}
        if "row_softmax" in self.ops:
            out["row_softmax_ms"] = self.timed(lambda: self.run_op("row_softmax", None), reps)
            for f in feats:
                out[f]["attention_fused_ms"] = self.timed(lambda: self.tcg.attention(self.meta, self.Xd[f], Y=self.Y), reps)
            out["attention_three_calls_ms"] = self.timed(
                lambda: [self.run_op(op, self.Xd[self.feat]) for op in self.ops], reps)
        return out

    def errors(self):
        """Largest normalised error of every operation of the step against the oracle, on the full outputs."""
        import numpy as np
        import oracle
        torch, tcg, g = self.torch, self.tcg, self.g
        rp, ci = (self.rp.cpu().numpy(), self.ci.cpu().numpy()) if self.perm is not None else (g.row_ptr, g.col_idx)
        x = self.Xd[self.feat]
        Xh = x.float().cpu().numpy()
        w = self.w_given.cpu().numpy() if self.w_given is not None else None
        out = {}
        if "sddmm" in self.ops:
            e = tcg.sddmm(self.meta, x)
            e_ref = oracle.sddmm(rp, ci, Xh)
            out["sddmm"] = norm_err(e.cpu().numpy(), e_ref)
            if "row_softmax" in self.ops:
                p = tcg.row_softmax(self.meta, e)
                out["row_softmax"] = norm_err(p.cpu().numpy(), oracle.row_softmax(rp, e.cpu().numpy().astype(np.float64)))
                w = p.cpu().numpy()
                Yg = tcg.spmm(self.meta, x, p)
            else:
                Yg = tcg.spmm(self.meta, x, self.w_given)
        else:
            Yg = tcg.spmm(self.meta, x, self.w_given)
        torch.cuda.synchronize()
        out["spmm"] = norm_err(Yg.cpu().numpy(), oracle.spmm(rp, ci, Xh, w))
        return out

    def name(self):
        c = self.c
        return ("config %s (%s): N=%d, %d stored entries, X %s N x %d, %s edge values, window %d x 8; "
                "step = sgt_build + %s" % (self.workload, c["name"], self.N, self.nnz, self.feat, self.D,
                                           "given" if self.weighted else "unit", self.H, " + ".join(self.ops)))

    def free(self):
        if self.meta is not None:
            self.meta.free()
            self.meta = None


def config_record(workload, feat, reorder, args):
    """One entry of `configs`: a few steps of a workload, its steady-state kernels and its error vs the oracle."""
    run = Run(workload, feat, args, reorder=reorder)
    ms_step, parts = run.steps(max(3, min(args.steps, 5)), 1)
    rec = {"workload": run.name() + (" [rows clustered first, %d rounds]" % reorder if reorder is not None else ""),
           "features": run.feat, "N": run.N, "D": run.D, "ms_per_step": ms_step, "step_parts_ms": parts}
    rec.update(run.sizes())
    rec["bytes"] = run.byte_counts(run.feat)
    st = run.steady(10, [run.feat])
    rec["steady_state"] = st
    sp = st[run.feat]["spmm_ms"]["median"]
    rec["spmm_gflops"] = 2.0 * run.nnz * run.D / sp / 1e6
    rec["sddmm_gedges_per_s"] = run.nnz / st[run.feat]["sddmm_ms"]["median"] / 1e6
    rec["spmm_frac_hbm_algorithmic"] = st[run.feat]["spmm_frac_hbm_algorithmic"]
    rec["spmm_frac_hbm_compulsory"] = rec["bytes"]["spmm_compulsory"] / (sp * 1e-3) / 1e9 / HBM_PEAK_GBS
    traffic, src = read_traffic(workload, run.feat) if reorder is None else (None, "no counter summary")
    rec["spmm_frac_hbm_counter"] = traffic / (sp * 1e-3) / 1e9 / HBM_PEAK_GBS if traffic else None
    if run.reorder_info is not None:
        run.reorder_info["window_unique_after"] = run.meta.total_unique
        rec["reorder"] = run.reorder_info
    rec["max_norm_err_vs_oracle"] = run.errors()
    run.free()
    del run
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None, choices=sorted(WORKLOADS),
                    help="run this workload alone (default: workload 4 as the headline, then every other one)")
    ap.add_argument("--features", default=None, choices=["f32", "bf16"])
    ap.add_argument("--nodes", type=int, default=None, help="override the node count of the workload")
    ap.add_argument("--dim", type=int, default=None, help="override the feature width of the workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="headline workload only")
    ap.add_argument("--backward", action="store_true",
                    help="also time the backward-pass building blocks (transpose, dX = A^T dY, dw = SDDMM(dY, X))")
    ap.add_argument("--window-height", type=int, default=16,
                    help="rows per window of the translation (16 as in the paper; 32 halves the neighbour fetches "
                         "of the MFMA tile path on clustered graphs)")
    ap.add_argument("--reorder", type=int, default=None, metavar="ROUNDS",
                    help="cluster the rows (tcg_reorder_rows with this many refinement rounds) and relabel the "
                         "graph and X before the timed steps; the one-off cost is reported under 'reorder'")
    ap.add_argument("--model", default=None, choices=["gcn", "agnn"],
                    help="also time training epochs of the paper's GCN (2 layers, 16 hidden) or AGNN (4 layers, "
                         "32 hidden) model built from the layer module on this workload's graph")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 512 MiB device copy (reference dispatch for HBM counter scaling)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2112_02052_amd as tcg

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    tcg.load_library()
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    workload = args.workload or "4"
    run = Run(workload, args.features, args, reorder=args.reorder)
    feat, ops = run.feat, run.ops
    N, nnz, D, g = run.N, run.nnz, run.D, run.g
    ms_per_step, parts = run.steps(args.steps, args.warmup)
    meta = run.meta
    spmm_ms, sddmm_ms = parts["spmm"], parts.get("sddmm")
    sizes = run.sizes()
    reps = max(5, args.steps)
    feats = ["f32", "bf16"]
    steady = run.steady(reps, feats)
    flops = 2.0 * nnz * D

    # The operations of a step (without the translation) as one HIP graph launch against the same calls issued
    # one by one: what a training loop gains from capturing them on the launch-bound workloads.
    def all_ops():
        for op in ops:
            run.run_op(op, run.Xd[feat])

    steady["ops_eager_ms"] = run.timed_loop(all_ops, reps)
    try:
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                all_ops()
        torch.cuda.synchronize()
        steady["ops_graph_replay_ms"] = run.timed_loop(graph.replay, reps)
        del graph
    except Exception as exc:                                   # a graph is a convenience here, not the product
        steady["ops_graph_replay_ms"] = None
        print("graph capture skipped: %s" % exc, file=sys.stderr)

    # Workloads whose X and Y fit in the last-level cache: the same calls rotating over enough copies of X
    # and Y that every call finds them cold (about 1 GB in total, beyond L2 and the 256 MB memory-side cache).
    copy_bytes = N * D * (SX[feat] + 4)
    if copy_bytes < (256 << 20):
        n_copies = int(min(64, max(2, (1 << 30) // max(copy_bytes, 1))))
        Xs = [run.Xd[feat].clone() for _ in range(n_copies)]
        Ys = [torch.empty_like(run.Y) for _ in range(n_copies)]
        turn = [0]

        def cold(op):
            k = turn[0] % n_copies
            turn[0] += 1
            if op == "sddmm":
                tcg.sddmm(meta, Xs[k], out=run.E)
            else:
                tcg.spmm(meta, Xs[k], run.P if op == "spmm_w" else run.w_given, Y=Ys[k])

        steady["cold_copies"] = n_copies
        steady["spmm_%s_cold_ms" % feat] = run.timed_loop(lambda: cold(run.spmm_op), max(reps, 2 * n_copies))
        steady["sddmm_%s_cold_ms" % feat] = run.timed_loop(lambda: cold("sddmm"), max(reps, 2 * n_copies))
        del Xs, Ys

    b = run.byte_counts(feat)
    b_spmm, b_sddmm = b["spmm_algorithmic"], b["sddmm_algorithmic"]
    t_launch = spmm_ms["mean"] * 1e-3                       # average launch duration over the timed region
    achieved = b_spmm / t_launch / 1e9
    tile_share = sizes["tile_edge_share"] if feat != "f32" else 0.0
    kernel = ("tcg_spmm (spmm_tile_direct_kernel)" if tile_share > 0.5
              else "tcg_spmm (spmm_gather_kernel + spmm_reduce_long_kernel)")
    traffic, traffic_src = read_traffic(workload, feat) if args.reorder is None else (None, "no counter summary")

    out = {
        "metric": METRIC,
        "value": flops / (spmm_ms["median"] * 1e-3) / 1e9,
        "unit": "GFLOP/s (useful, SpMM)",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": feat,
        "data": "synthetic",
        "config": dict({"workload": run.name(), "features": feat}, **sizes),
        "step_parts_ms": parts,
        "spmm_hbm_gbs_algorithmic": achieved,
        "sgt_medges_per_s": nnz / (parts["sgt_build"]["median"] * 1e-3) / 1e6,
        "steady_state": steady,
        "roofline": {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "frac_is": "algorithmic bytes of the method (every window-unique neighbour row once) per launch "
                                "/ average launch duration / peak; the kernels' caches serve rows shared between "
                                "windows, so this can exceed the HBM traffic and 1 -- frac_counter is the measured one",
                     "traffic": traffic,
                     "traffic_source": traffic_src,
                     # HBM-side bytes counted by rocprofv3 for the same launch / average launch duration / peak
                     # (FETCH_SIZE counts L2 misses; some are served by the memory-side cache: an upper bound)
                     "hbm_gbs_counter": traffic / t_launch / 1e9 if traffic else None,
                     "frac_counter": traffic / t_launch / 1e9 / HBM_PEAK_GBS if traffic else None,
                     "algorithmic_bytes": b_spmm,
                     "compulsory_bytes": b["spmm_compulsory"],
                     # the same launch priced with every X row once: what memory has to deliver at least
                     "frac_compulsory": b["spmm_compulsory"] / t_launch / 1e9 / HBM_PEAK_GBS,
                     "csr_gather_bytes": b["spmm_csr_gather"]},
        "generate_s": run.gen_s,
    }
    # Throughput against the feature width on the same graph (the paper's embedding-dimension study, section 5.4):
    # D = 16 .. 256 in both feature types, a few calls each on the reused translation; timing only (uniform
    # features from a seeded generator on the device).
    if not args.no_configs and args.model is None and not args.backward:
        gen = torch.Generator(device=dev)
        gen.manual_seed(0)
        tdt = {"f32": torch.float32, "bf16": torch.bfloat16}
        sweep = []
        for d in (16, 32, 64, 128, 256):
            x32 = torch.rand((g.n_cols, d), generator=gen, device=dev) * 2.0 - 1.0
            y = torch.empty((N, d), dtype=torch.float32, device=dev)
            for f in feats:
                x = x32.to(tdt[f])
                sp = run.timed(lambda: tcg.spmm(meta, x, run.P if run.spmm_op == "spmm_w" else run.w_given, Y=y), 6)
                sd = run.timed(lambda: tcg.sddmm(meta, x, out=run.E), 6)
                b_alg = algorithmic_bytes_spmm(N, nnz, meta.total_unique, meta.n_windows, d, SX[f], 4, run.weighted)
                sweep.append({"D": d, "features": f, "spmm_ms": sp["median"], "sddmm_ms": sd["median"],
                              "spmm_gflops": 2.0 * nnz * d / sp["median"] / 1e6,
                              "sddmm_gedges": nnz / sd["median"] / 1e6,
                              "spmm_frac_hbm_algorithmic": b_alg / (sp["median"] * 1e-3) / 1e9 / HBM_PEAK_GBS})
            del x32, y
        out["d_sweep"] = sweep
    if run.reorder_info is not None:
        run.reorder_info["window_unique_after"] = meta.total_unique
        out["reorder"] = run.reorder_info
    if sddmm_ms is not None:
        out["sddmm_gedges_per_s"] = nnz / (sddmm_ms["median"] * 1e-3) / 1e9
        out["sddmm_hbm_gbs_algorithmic"] = b_sddmm / (sddmm_ms["mean"] * 1e-3) / 1e9
    out["max_norm_err_vs_oracle"] = None

    if args.backward:
        def once(fn):
            a, b2 = run.ev(), run.ev()
            a.record()
            r = fn()
            b2.record()
            torch.cuda.synchronize()
            return r, a.elapsed_time(b2)
        rp, ci = run.rp, run.ci
        tdt = {"f32": torch.float32, "bf16": torch.bfloat16}
        tcg.csr_transpose(rp, ci, g.n_cols)                              # warm-up (fills the allocator cache)
        (rpt, cit, perm), tr_ms = once(lambda: tcg.csr_transpose(rp, ci, g.n_cols))
        meta_t, sgt_t_ms = once(lambda: tcg.sgt_build(rpt, cit, run.H, run.TW, n_cols=N, validate=False))
        Gd = torch.randn((N, D), device=dev).to(tdt[feat])               # stands for dL/dY
        w_fwd = run.w_given if run.w_given is not None else torch.ones(nnz, device=dev)
        w_t = tcg.edge_gather(perm, w_fwd)
        out["backward"] = {
            "csr_transpose_ms": tr_ms, "sgt_build_transposed_ms": sgt_t_ms,
            "csr_transpose_steady_ms": run.timed(lambda: tcg.csr_transpose(rp, ci, g.n_cols), 5),
            "edge_gather_ms": run.timed_loop(lambda: tcg.edge_gather(perm, w_fwd, out=w_t), reps),
            "dX_spmm_transposed_ms": run.timed_loop(lambda: tcg.spmm(meta_t, Gd, w_t, Y=run.Y), reps),
            "dw_sddmm_pq_ms": run.timed_loop(lambda: tcg.sddmm_pq(meta, Gd, run.Xd[feat], out=run.E), reps),
        }
        meta_t.free()

    if args.model:
        import paper_2112_02052_amd.nn as tnn
        graph = tnn.TiledGraph(run.rp, run.ci, window_h=run.H, validate=False)
        graph.transposed()                                                # built once, like the forward plan
        torch.manual_seed(0)
        n_classes = 10
        Xf = run.Xd["f32"]
        if args.model == "gcn":
            model = tnn.GCN(D, 16, n_classes).to(dev)
            wv = run.w_given if run.w_given is not None else None
            fwd = lambda: model(Xf, graph, wv)                            # noqa: E731
        else:
            model = tnn.AGNN(D, 32, n_classes, n_layers=4).to(dev)
            fwd = lambda: model(Xf, graph)                                # noqa: E731
        labels = torch.randint(0, n_classes, (N,), device=dev)
        opt = torch.optim.Adam(model.parameters(), lr=0.01)

        def epoch():
            opt.zero_grad(set_to_none=True)
            loss = -fwd().gather(1, labels[:, None]).mean()               # negative log-likelihood of the labels
            loss.backward()
            opt.step()

        def forward_only():
            with torch.no_grad():
                fwd()

        for _ in range(3):
            epoch()
        out["model"] = {"name": args.model, "layers": 2 if args.model == "gcn" else 4,
                        "hidden": 16 if args.model == "gcn" else 32, "in_dim": D, "classes": n_classes,
                        "epoch_ms": run.timed_loop(epoch, reps), "forward_ms": run.timed_loop(forward_only, reps),
                        "epoch": "forward + NLL loss + backward + Adam step, fp32, translated graph and its transpose reused"}
        graph.free()

    if not args.no_cpu_baseline:
        import oracle
        out["max_norm_err_vs_oracle"] = run.errors()
        rp_h, ci_h = (run.rp.cpu().numpy(), run.ci.cpu().numpy()) if run.perm is not None else (g.row_ptr, g.col_idx)
        Xh = run.Xd[feat].float().cpu().numpy()
        w_cpu = run.w_given.cpu().numpy() if run.w_given is not None else None
        if "spmm_w" in ops:
            w_cpu = run.P.cpu().numpy()
        cores = oracle.num_threads()

        def cpu_time(fn, budget_s, at_least=3, at_most=30):
            fn()                                                       # warm-up
            ts = []
            end = time.perf_counter() + budget_s
            while len(ts) < at_least or (time.perf_counter() < end and len(ts) < at_most):
                t1 = time.perf_counter()
                fn()
                ts.append(time.perf_counter() - t1)
            return sorted(ts)[len(ts) // 2], len(ts)

        t_cpu, n_cpu = cpu_time(lambda: oracle.spmm(rp_h, ci_h, Xh, w_cpu), 2.0)
        t_f32, n_f32 = cpu_time(lambda: oracle.spmm_f32acc(rp_h, ci_h, Xh, w_cpu), 2.0)
        t_sd, n_sd = cpu_time(lambda: oracle.sddmm_f32acc(rp_h, ci_h, Xh), 2.0)
        t_sgt_par, n_sgt = cpu_time(lambda: oracle.sgt(rp_h, ci_h, run.H, run.TW, parallel=True), 2.0, at_most=5)
        t1 = time.perf_counter()
        oracle.sgt(rp_h, ci_h, run.H, run.TW)
        t_sgt_seq = time.perf_counter() - t1
        whole = "the full workload (all %d rows)" % N
        out["cpu_baseline"] = {"value": flops / t_cpu / 1e9, "unit": "GFLOP/s (useful, SpMM)", "cores": cores,
                               "kind": "oracle",
                               "sample": "%s, the parity oracle (double accumulation, CSR order), median of %d runs, "
                                         "%.3f s each" % (whole, n_cpu, t_cpu)}
        out["cpu_baseline_f32acc"] = {"value": flops / t_f32 / 1e9, "unit": "GFLOP/s (useful, SpMM)", "cores": cores,
                                      "kind": "oracle variant with float accumulation (timing only)",
                                      "sample": "%s, median of %d runs, %.3f s each" % (whole, n_f32, t_f32)}
        out["cpu_baseline_sddmm"] = {"value": nnz / t_sd / 1e9, "unit": "G edges/s (SDDMM)", "cores": cores,
                                     "kind": "oracle variant with float accumulation (timing only)",
                                     "sample": "%s, median of %d runs, %.3f s each" % (whole, n_sd, t_sd)}
        out["cpu_baseline_sgt"] = {"value": nnz / t_sgt_par / 1e6, "unit": "M stored entries/s (translation)",
                                   "cores": cores, "kind": "oracle, windows spread over the cores (same results)",
                                   "sample": "%s, median of %d runs, %.3f s each" % (whole, n_sgt, t_sgt_par),
                                   "sequential": {"value": nnz / t_sgt_seq / 1e6, "cores": 1,
                                                  "sample": "Algorithm 1 window after window, one run, %.3f s" % t_sgt_seq}}
    if args.calibrate_copy:
        src = torch.empty(128 << 20, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                                            # reads 512 MiB, writes 512 MiB
        torch.cuda.synchronize()
    run.free()
    del run
    tcg.release_cached_memory()

    if args.workload is None and not args.no_configs:
        torch.cuda.empty_cache()
        configs = []
        for wl, f, reorder in OTHER_CONFIGS:
            configs.append(config_record(wl, f, reorder, args))
            tcg.release_cached_memory()
            torch.cuda.empty_cache()
        out["configs"] = configs
    print(json.dumps(out))


if __name__ == "__main__":
    main()
