"""GPU parity: the HIP library (through its C ABI binding) against the CPU oracle, element by
element on the same seeded inputs.  Integer metadata must be bit-exact; floats within the
stated normalised tolerances."""
import numpy as np
import pytest
import torch

import oracle
import paper_2112_02052_amd as tcg
import workloads as W
from workloads.graphs import CSR

from gpu_util import TORCH_DT, TOL_F32, TOL_MFMA, check_sgt, dev, norm_err, upload_csr, upload_x

pytestmark = pytest.mark.gpu


def csr_from_rows(rows, n_cols):
    rp = np.zeros(len(rows) + 1, dtype=np.int32)
    rp[1:] = np.cumsum([len(r) for r in rows])
    ci = np.concatenate([np.asarray(r, dtype=np.int32) for r in rows]) if rp[-1] else np.zeros(0, np.int32)
    return CSR(len(rows), n_cols, rp, ci)


def hub_graph(n=3000, seed=5):
    """Rows of very different lengths: two hub rows (large-window class of SGT, many segments),
    a mid-size row (medium class), empty rows, shuffled column order and one repeated entry."""
    rng = np.random.default_rng(seed)
    rows = []
    for i in range(n):
        if i == 7:
            k = 6000
        elif i == 1500:
            k = 2500
        elif i == 40:
            k = 1500
        elif i % 11 == 0:
            k = 0
        else:
            k = int(rng.integers(1, 40))
        k = min(k, n)
        rows.append(rng.permutation(n)[:k])
    rows[3] = np.concatenate([rows[3], rows[3][:1]])      # a repeated (row, col) entry
    return csr_from_rows(rows, n)


# ----------------------------------------------------------------------------------------------
# SGT: bit-exact metadata
# ----------------------------------------------------------------------------------------------

@pytest.mark.parametrize("cfg,n,H,W_", [
    (1, 2048, 16, 8), (1, 2048, 16, 16), (2, 20000, 16, 8), (3, 20000, 16, 16), (4, 50000, 16, 32),
    (5, 64 * 200, 16, 16), (4, 1003, 12, 5), (3, 5000, 1, 8), (2, 777, 777, 4), (1, 100, 128, 8),
])
def test_sgt_bit_exact(cfg, n, H, W_):
    g = W.make_config(cfg, n=n, d=4)["csr"]
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, H, W_)
    check_sgt(meta, g, H, W_)
    meta.free()


def test_sgt_all_size_classes_and_unsorted_rows():
    g = hub_graph()
    rp, ci = upload_csr(g)
    for H, W_ in ((16, 8), (4, 16), (64, 8)):
        meta = tcg.sgt_build(rp, ci, H, W_)
        ref = check_sgt(meta, g, H, W_)
        assert np.diff(ref["win_unique_ptr"]).max() > 1024
        meta.free()


def test_sgt_large_windows_in_both_bitmap_variants():
    # Windows above 4096 entries use a bitmap over the column space: in LDS when the column space fits
    # (up to about 1.12 M columns), in device memory beyond.  Both with columns up to the last one, rows
    # in shuffled order, repeated entries, and a window that is nearly full.
    rng = np.random.default_rng(21)
    for n_cols in (70000, 1120000 - 7, 1400003):
        rows = []
        for i in range(48):
            k = 400 if i < 16 else (3 if i < 32 else 700)
            r = rng.integers(0, n_cols, size=k)
            if i == 0:
                r[:3] = (0, n_cols - 1, n_cols - 1)
            rows.append(r)
        g = csr_from_rows(rows, n_cols)
        rp, ci = upload_csr(g)
        meta = tcg.sgt_build(rp, ci, 16, 8, n_cols=n_cols)
        check_sgt(meta, g, 16, 8)
        meta.free()


@pytest.mark.parametrize("x_dtype,D", [("f32", 128), ("f32", 192), ("bf16", 384)])
def test_wide_rows_of_a_large_operand_are_gathered_in_feature_slabs(x_dtype, D):
    # Rows of 512 bytes and more of an operand beyond 64 MB are gathered in 256-byte slabs, one launch per slab
    # (the aggregation writes each slab's columns, the edge scores add up over the slabs): 2, 3 and 3 slabs here,
    # with edge values, against the oracle.
    c = W.make_config(4, n=140000, d=D, x_dtype=x_dtype)
    g, X = c["csr"], c["X"]
    assert g.n_cols * D * (4 if x_dtype == "f32" else 2) >= 64 << 20
    rng = np.random.default_rng(3)
    w = rng.uniform(0.5, 1.5, g.nnz).astype(np.float32)
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    Xd = upload_x(X, x_dtype)
    Y = tcg.spmm(meta, Xd, torch.from_numpy(w).to(dev()))
    e = tcg.sddmm(meta, Xd)
    torch.cuda.synchronize()
    assert norm_err(Y.cpu().numpy(), oracle.spmm(g.row_ptr, g.col_idx, X, w)) <= TOL_F32
    assert norm_err(e.cpu().numpy(), oracle.sddmm(g.row_ptr, g.col_idx, X)) <= TOL_F32
    e2 = tcg.sddmm(meta, Xd, out=torch.full_like(e, float("nan")))        # what is in the output beforehand is not used
    torch.cuda.synchronize()
    assert torch.equal(e, e2)
    meta.free()


def test_more_windows_than_one_workgroup_scans():
    # Above 16,384 windows the unique counts are scanned, and the windows' paths chosen, by a multi-workgroup pass
    # instead of the single workgroup that serves smaller graphs: a clustered graph of 19,200 windows whose windows
    # go to the MFMA tile path (translation, plan statistics, SpMM and SDDMM), and one-row windows on a power-law
    # graph.
    c = W.make_config(5, n=64 * 4800, permute=False, d=64)
    g, X = c["csr"], c["X"]
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    assert meta.n_windows == 19200
    ref = check_sgt(meta, g, 16, 8)
    uw = np.diff(ref["win_unique_ptr"])
    nnz_w = np.add.reduceat(np.diff(g.row_ptr), np.arange(0, g.n_rows, 16))
    expect = int(np.sum((uw > 0) & (uw <= 512) & (nnz_w >= 2.0 * uw)))
    assert tcg.sgt_plan_stats(meta)["n_tile_windows"] == expect and expect > 0.95 * meta.n_windows
    Xd = upload_x(X, "bf16")
    e = tcg.sddmm(meta, Xd)
    Y = tcg.spmm(meta, Xd)
    torch.cuda.synchronize()
    assert norm_err(e.cpu().numpy(), oracle.sddmm(g.row_ptr, g.col_idx, X)) <= TOL_F32
    assert norm_err(Y.cpu().numpy(), oracle.spmm(g.row_ptr, g.col_idx, X)) <= TOL_F32
    meta.free()
    g = W.make_config(3, n=30000, d=4)["csr"]
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 1, 8)
    assert meta.n_windows == 30000
    check_sgt(meta, g, 1, 8)
    meta.free()


def test_sgt_hub_windows_translated_in_parts():
    # A window of the LDS-bitmap class with more than 16,384 entries is listed in 2 .. 8 parts (each part ranks
    # its share of the entries): windows in 2, 3 and 8 parts (the last beyond 8 x 16,384 entries) next to ordinary
    # ones, unsorted rows with repeated entries, the first and the last column present.
    rng = np.random.default_rng(33)
    n_cols = 300000
    per_row = [1200] * 16 + [5] * 16 + [2900] * 16 + [40] * 16 + [9000] * 16 + [700] * 16
    rows = [rng.integers(0, n_cols, size=k) for k in per_row]
    rows[0][:2] = (0, n_cols - 1)
    rows[64][:4] = (n_cols - 1, 0, 7, 7)
    g = csr_from_rows(rows, n_cols)
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8, n_cols=n_cols)
    check_sgt(meta, g, 16, 8)
    meta.free()
    # 12 rows per window: parts whose shares do not divide evenly
    meta = tcg.sgt_build(rp, ci, 12, 16, n_cols=n_cols)
    check_sgt(meta, g, 12, 16)
    meta.free()


@pytest.mark.parametrize("cfg,n,H", [(1, 2048, 16), (3, 30000, 16), (4, 50000, 16), (5, 64 * 100, 16), (2, 1003, 12)])
def test_sgt_tile_counts_with_and_without_the_translation(cfg, n, H):
    # Section 5.2's quantity for the paper's two tile widths (8: aggregation, 16: edge features) and two
    # others, from one translated graph; bit-exact against the oracle's count from the CSR.
    g = W.make_config(cfg, n=n, d=4)["csr"]
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, H, 8)
    for tile_w in (8, 16, 1, 5):
        assert tcg.sgt_tile_stats(meta, tile_w) == oracle.tile_counts(g.row_ptr, g.col_idx, H, tile_w), tile_w
    assert tcg.sgt_tile_stats(meta, 8)[0] == meta.total_tiles
    meta.free()


def test_sgt_empty_and_degenerate():
    for g in (CSR(0, 0, np.zeros(1, np.int32), np.zeros(0, np.int32)),
              CSR(37, 37, np.zeros(38, np.int32), np.zeros(0, np.int32)),
              csr_from_rows([[0]], 1),
              csr_from_rows([[], [5, 2], []] + [[]] * 30 + [[9]], 10)):
        rp, ci = upload_csr(g)
        meta = tcg.sgt_build(rp, ci, 16, 8, n_cols=g.n_cols)
        check_sgt(meta, g, 16, 8)
        X = torch.ones((max(g.n_cols, g.n_rows, 1), 4), device=dev())
        Y = tcg.spmm(meta, X)
        e = tcg.sddmm(meta, X)
        torch.cuda.synchronize()
        assert Y.shape == (g.n_rows, 4) and e.numel() == g.nnz
        if g.n_rows:
            assert np.array_equal(Y.cpu().numpy()[:, 0], np.diff(g.row_ptr).astype(np.float32))
        meta.free()


def test_out_of_device_memory_is_an_error_code_and_leaves_the_plan_usable():
    # Scratch for an absurd feature width (1,600 split-row segments x 2^31 - 1 columns x 4 bytes = 13 TB) cannot be
    # allocated: TCG_ENOMEM, and the plan, its scratch and the library keep working.
    rng = np.random.default_rng(2)
    rows = [np.sort(rng.choice(250000, size=k, replace=False)) for k in (200000, 3, 0, 900)] + [[i] for i in range(60)]
    g = csr_from_rows(rows, 250000)
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8, n_cols=g.n_cols)
    X = rng.standard_normal((g.n_cols, 16)).astype(np.float32)
    Xd = torch.from_numpy(X).to(dev())
    Y0 = tcg.spmm(meta, Xd)
    with pytest.raises(tcg.TcgError) as ei:
        tcg.sgt_reserve(meta, 2 ** 31 - 1)
    assert ei.value.status == -4
    Y1 = tcg.spmm(meta, Xd)
    torch.cuda.synchronize()
    assert torch.equal(Y0, Y1)
    assert norm_err(Y1.cpu().numpy(), oracle.spmm(g.row_ptr, g.col_idx, X, None)) <= TOL_F32
    meta.free()


def test_builds_and_calls_from_two_host_threads():
    # Two host threads, each with its own stream, translate different graphs and run the aggregation at the same
    # time (the translations share the library's two side streams and its allocator): every result is checked
    # against the oracle, and the translations bit for bit.
    import threading
    cases = [(W.make_config(3, n=20000, d=32), 16), (W.make_config(4, n=30000, d=64), 16),
             (W.make_config(2, n=6000, d=16), 12), (W.make_config(5, n=64 * 150, d=64, permute=False), 16)]
    refs = [(oracle.sgt(c["csr"].row_ptr, c["csr"].col_idx, H, 8),
             oracle.spmm(c["csr"].row_ptr, c["csr"].col_idx, np.asarray(c["X"], dtype=np.float32), None)) for c, H in cases]
    errors = []

    def work(tid):
        try:
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for rep in range(4):
                    for k in range(tid, len(cases), 2):
                        (c, H), (sref, yref) = cases[k], refs[k]
                        g = c["csr"]
                        rp, ci = upload_csr(g)
                        meta = tcg.sgt_build(rp, ci, H, 8)
                        got = {n: v.cpu().numpy() for n, v in tcg.sgt_export(meta).items()}
                        for n in ("win_partition", "edge_to_col", "col_to_row"):
                            assert np.array_equal(got[n], sref[n]), (k, n)
                        Y = tcg.spmm(meta, upload_x(np.asarray(c["X"], dtype=np.float32), "f32"))
                        stream.synchronize()
                        assert norm_err(Y.cpu().numpy(), yref) <= TOL_F32, k
                        meta.free()
        except BaseException as exc:        # reported by the main thread
            errors.append((tid, repr(exc)))

    threads = [threading.Thread(target=work, args=(t,)) for t in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


def test_calls_that_wait_for_the_stream_refuse_a_stream_under_capture():
    # Translation, policy change, tile statistics and export to the host wait for the stream; under HIP graph
    # capture they return TCG_ECAPTURE before they touch it, so the capture goes on and the graph replays.
    c = W.make_config(2, n=3000, d=16)
    g, X = c["csr"], c["X"]
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    Xd = upload_x(X, "f32")
    Y = torch.empty((g.n_rows, 16), device=dev())
    tcg.spmm(meta, Xd, Y=Y)
    torch.cuda.synchronize()
    Y_eager = Y.clone()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    refused = []
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for call in (lambda: tcg.sgt_build(rp, ci, 16, 8), lambda: tcg.sgt_set_policy(meta, tcg.POLICY_GATHER),
                         lambda: tcg.sgt_tile_stats(meta, 8), lambda: tcg.csr_transpose(rp, ci)):
                with pytest.raises(tcg.TcgError) as ei:
                    call()
                refused.append(ei.value.status)
            tcg.spmm(meta, Xd, Y=Y)
    assert refused == [-7] * 4
    Y.zero_()
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(Y, Y_eager)
    meta.free()


def test_sgt_rejects_malformed_csr():
    rp = torch.tensor([0, 2, 1, 3], dtype=torch.int32, device=dev())
    ci = torch.tensor([0, 1, 2], dtype=torch.int32, device=dev())
    with pytest.raises(tcg.TcgError) as ei:
        tcg.sgt_build(rp, ci, 16, 8)
    assert ei.value.status == -2
    rp = torch.tensor([0, 1, 2, 3], dtype=torch.int32, device=dev())
    ci = torch.tensor([0, 3, 2], dtype=torch.int32, device=dev())      # column 3 of a 3-column matrix
    with pytest.raises(tcg.TcgError) as ei:
        tcg.sgt_build(rp, ci, 16, 8)
    assert ei.value.status == -2
    with pytest.raises(tcg.TcgError) as ei:
        tcg.sgt_build(rp, torch.tensor([0, 1, 2], dtype=torch.int32, device=dev()), 0, 8)
    assert ei.value.status == -1
    meta = tcg.sgt_build(rp, torch.tensor([0, 1, 2], dtype=torch.int32, device=dev()), 8, 8)
    with pytest.raises(tcg.TcgError) as ei:
        tcg.sgt_set_policy(meta, tcg.POLICY_TILE)                       # tile path needs window height 16 or 32
    assert ei.value.status == -1
    meta.free()


def test_cached_memory_is_reused_and_can_be_released():
    # Buffers of a freed translation go back to the library's cache; a later build (which may get
    # them, stale contents included) must still be bit-exact, also after the cache was released.
    g1 = W.make_config(4, n=20000, d=4)["csr"]
    g2 = W.make_config(3, n=15000, d=4)["csr"]
    for rnd in range(3):
        for g in (g1, g2):
            rp, ci = upload_csr(g)
            meta = tcg.sgt_build(rp, ci, 16, 8)
            check_sgt(meta, g, 16, 8)
            meta.free()
        if rnd == 1:
            tcg.release_cached_memory()


# ----------------------------------------------------------------------------------------------
# SpMM
# ----------------------------------------------------------------------------------------------

def run_spmm_case(g, X, x_dtype, w, policy, tol, H=16, y_dtype=torch.float32, pad=0):
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, H, 8, n_cols=g.n_cols)
    tcg.sgt_set_policy(meta, policy)
    Xd = upload_x(X, x_dtype)
    if pad:                                                # leading dimension larger than D
        big = torch.zeros((Xd.shape[0], Xd.shape[1] + pad), dtype=Xd.dtype, device=dev())
        big[:, :Xd.shape[1]] = Xd
        Xd = big[:, :X.shape[1]]
    wd = torch.from_numpy(w).to(dev()) if w is not None else None
    Y = torch.full((g.n_rows, X.shape[1]), float("nan"), dtype=y_dtype, device=dev())
    tcg.spmm(meta, Xd, wd, Y=Y)
    torch.cuda.synchronize()
    ref = oracle.spmm(g.row_ptr, g.col_idx, X, w)
    err = norm_err(Y.to(torch.float32).cpu().numpy(), ref)
    stats = tcg.sgt_plan_stats(meta)
    meta.free()
    assert err <= tol, "normalised error %.3g above %.1g" % (err, tol)
    return stats


@pytest.mark.parametrize("cfg,n,D", [(1, 2048, 16), (2, 20000, 64), (3, 20000, 32), (4, 30000, 128),
                                     (4, 5000, 256), (2, 3000, 48), (2, 3000, 5), (1, 500, 1),
                                     (3, 4000, 320), (3, 3000, 1024 + 64)])
def test_spmm_fp32_gather(cfg, n, D):
    c = W.make_config(cfg, n=n, d=D)
    w = c["w"]
    if w is None:
        w = np.random.default_rng(1).standard_normal(c["csr"].nnz).astype(np.float32)
    run_spmm_case(c["csr"], c["X"], "f32", w, tcg.POLICY_AUTO, TOL_F32)
    run_spmm_case(c["csr"], c["X"], "f32", None, tcg.POLICY_GATHER, TOL_F32)


@pytest.mark.parametrize("D", [4, 8, 16])
def test_spmm_narrow_result_of_split_rows(D):
    """Split rows whose partial sums are added by the one-wavefront-per-row kernel (4, 8, 16 columns), with and
    without edge values, fp32 and 16-bit results."""
    g = hub_graph()
    X = W.features_normal(g.n_cols, D, 5)
    w = np.random.default_rng(3).standard_normal(g.nnz).astype(np.float32)
    stats = run_spmm_case(g, X, "f32", w, tcg.POLICY_GATHER, TOL_F32)
    assert stats["n_long_rows"] > 0
    run_spmm_case(g, X, "f32", None, tcg.POLICY_GATHER, TOL_F32)
    run_spmm_case(g, X, "f32", None, tcg.POLICY_GATHER, 2.0 ** -8, y_dtype=torch.bfloat16)


def test_spmm_fp32_strided_and_other_window_heights():
    c = W.make_config(4, n=6000, d=64)
    run_spmm_case(c["csr"], c["X"], "f32", None, tcg.POLICY_AUTO, TOL_F32, pad=8)
    run_spmm_case(c["csr"], c["X"], "f32", None, tcg.POLICY_AUTO, TOL_F32, pad=3)    # misaligned rows -> generic kernel
    run_spmm_case(c["csr"], c["X"], "f32", None, tcg.POLICY_AUTO, TOL_F32, H=7)
    g = hub_graph()
    X = W.features_normal(g.n_cols, 32, 3)
    w = np.random.default_rng(2).standard_normal(g.nnz).astype(np.float32)
    run_spmm_case(g, X, "f32", w, tcg.POLICY_AUTO, TOL_F32)


def test_spmm_closed_form_full_size_config2():
    # X[:, d] = sqrt(deg) is reproduced by the symmetric normalisation (see the oracle's pin).
    c = W.make_config(2, d=64)
    g = c["csr"]
    s = np.sqrt(g.degrees().astype(np.float64))
    X = np.repeat(s[:, None], 64, axis=1).astype(np.float32)
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    Y = tcg.spmm(meta, upload_x(X, "f32"), torch.from_numpy(c["w"]).to(dev()))
    torch.cuda.synchronize()
    np.testing.assert_allclose(Y.cpu().numpy(), X, rtol=3e-6)
    meta.free()


@pytest.mark.parametrize("x_dtype", ["bf16", "f16"])
@pytest.mark.parametrize("policy", [tcg.POLICY_GATHER, tcg.POLICY_TILE, tcg.POLICY_AUTO])
def test_spmm_16bit_features(x_dtype, policy):
    rnd = W.round_to_bf16 if x_dtype == "bf16" else (lambda a: a.astype(np.float16).astype(np.float32))
    for cfg, n, D, permute in ((5, 64 * 60, 256, False), (5, 64 * 30, 64, True), (3, 4000, 32, True),
                               (4, 3000, 128, True), (5, 64 * 10, 72, False)):
        c = W.make_config(cfg, n=n, d=D, permute=permute)
        X = rnd(c["X"])
        w = np.random.default_rng(3).uniform(0.5, 1.5, c["csr"].nnz).astype(np.float32)
        tol = TOL_F32 if policy == tcg.POLICY_GATHER else TOL_MFMA
        st = run_spmm_case(c["csr"], X, x_dtype, w, policy, tol)
        if policy == tcg.POLICY_TILE:
            assert st["nnz_tile"] == c["csr"].nnz
        if policy == tcg.POLICY_AUTO and cfg == 5 and not permute:
            assert st["n_tile_windows"] > 0.9 * (n // 16)       # clustered windows take the MFMA path
        run_spmm_case(c["csr"], X, x_dtype, None, policy, TOL_F32)   # unit weights are exact in 16 bits


@pytest.mark.parametrize("policy", [tcg.POLICY_TILE, tcg.POLICY_AUTO])
def test_spmm_fp32_features_on_the_tile_path(policy):
    # gfx950 has no MFMA with fp32 inputs: the tile kernel splits every fp32 operand exactly into three bf16
    # values and accumulates the six leading products in fp32, so the fp32 tolerance applies.
    for cfg, n, D, permute in ((5, 64 * 60, 256, False), (5, 64 * 30, 64, True), (3, 4000, 32, True),
                               (4, 3000, 128, True), (5, 64 * 10, 72, False), (5, 64 * 12, 300, False)):
        c = W.make_config(cfg, n=n, d=D, permute=permute)
        w = np.random.default_rng(3).uniform(0.5, 1.5, c["csr"].nnz).astype(np.float32)
        st = run_spmm_case(c["csr"], c["X"], "f32", w, policy, TOL_F32)
        if policy == tcg.POLICY_TILE:
            assert st["nnz_tile"] == c["csr"].nnz
        if policy == tcg.POLICY_AUTO and cfg == 5 and not permute:
            assert st["n_tile_windows"] > 0.9 * (n // 16)
        run_spmm_case(c["csr"], c["X"], "f32", None, policy, TOL_F32)


@pytest.mark.parametrize("D", [4, 12, 36, 68, 132, 200, 260, 516, 1024])
def test_spmm_fp32_tile_path_feature_widths(D):
    # One, two and four 64-feature blocks per wavefront, several feature parts, a ragged last block, padded
    # rows, outputs that cannot take 16-byte stores, and a 16-bit result.
    c = W.make_config(5, n=64 * 12, d=D, permute=False)
    g, X = c["csr"], c["X"]
    w = np.random.default_rng(D).standard_normal(g.nnz).astype(np.float32)
    run_spmm_case(g, X, "f32", w, tcg.POLICY_TILE, TOL_F32)
    run_spmm_case(g, X, "f32", None, tcg.POLICY_TILE, TOL_F32, pad=4)
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    tcg.sgt_set_policy(meta, tcg.POLICY_TILE)
    Xd = upload_x(X, "f32")
    ref = oracle.spmm(g.row_ptr, g.col_idx, X, None)
    for y_dtype, tol in ((torch.float32, TOL_F32), (torch.bfloat16, 2.0 ** -8)):
        big = torch.full((g.n_rows, D + 3), float("nan"), dtype=y_dtype, device=dev())
        Y = big[:, 1:D + 1]                                   # odd leading dimension, shifted start
        tcg.spmm(meta, Xd, None, Y=Y)
        torch.cuda.synchronize()
        assert norm_err(Y.to(torch.float32).cpu().numpy(), ref) <= tol
        assert torch.isnan(big[:, 0]).all() and torch.isnan(big[:, D + 1:]).all()   # nothing outside Y
    meta.free()


def test_spmm_fp32_tile_path_windows_with_many_edges():
    # 2 dense blocks per window: 512 edges, kept in LDS; 20: the whole condensed adjacency of the window in
    # LDS; 48: 768 condensed columns, which only a forced policy sends here (edges re-read per chunk).
    for blocks, D in ((2, 40), (20, 136), (48, 40)):
        g = W.dense_block_windows(1024, blocks, seed=5)
        X = W.features_normal(1024, D, 6)
        w = np.random.default_rng(blocks).standard_normal(g.nnz).astype(np.float32)
        run_spmm_case(g, X, "f32", None, tcg.POLICY_TILE, TOL_F32)
        run_spmm_case(g, X, "f32", w, tcg.POLICY_TILE, TOL_F32)


def test_spmm_fp32_tile_path_is_as_accurate_as_fp32_arithmetic():
    # The split into bf16 triples is exact and only products below 2^-23 of |w x| are dropped, so the error of an
    # output stays at the level of fp32 rounding relative to sum |w||x| of its row -- also for values whose
    # magnitudes differ by many binades, where a dropped or misplaced term of the split (2^-16 of a product)
    # would show at once.  The gather path (plain fp32 FMAs) is held to the same bound.
    c = W.make_config(5, n=64 * 60, d=256, permute=False)
    g = c["csr"]
    rng = np.random.default_rng(1)
    Xw = (rng.standard_normal((g.n_cols, 256)) * np.exp2(rng.integers(-20, 21, (g.n_cols, 256)))).astype(np.float32)
    ww = (rng.standard_normal(g.nnz) * np.exp2(rng.integers(-10, 11, g.nnz))).astype(np.float32)
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    for X, w in ((Xw, ww), (Xw, None), (c["X"], rng.uniform(0.5, 1.5, g.nnz).astype(np.float32))):
        ref = oracle.spmm(g.row_ptr, g.col_idx, X, w)
        mag = oracle.spmm(g.row_ptr, g.col_idx, np.abs(X), None if w is None else np.abs(w))
        for policy in (tcg.POLICY_GATHER, tcg.POLICY_TILE):
            tcg.sgt_set_policy(meta, policy)
            Y = tcg.spmm(meta, upload_x(X, "f32"), None if w is None else torch.from_numpy(w).to(dev()))
            torch.cuda.synchronize()
            rel = np.abs(Y.cpu().numpy().astype(np.float64) - ref) / np.maximum(mag, 1e-300)
            assert rel.max() <= 2.0 ** -19, (policy, rel.max())
    meta.free()


def test_spmm_integer_inputs_are_bit_exact_on_every_path():
    # Unit edge values and small-integer features: every product and fp32 partial sum is exact,
    # so any path must reproduce the oracle bit for bit whatever its summation order.
    g = hub_graph(2000)
    X = np.random.default_rng(0).integers(-8, 9, (g.n_cols, 64)).astype(np.float32)
    ref = oracle.spmm(g.row_ptr, g.col_idx, X)
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    for x_dtype, policy in (("f32", tcg.POLICY_GATHER), ("bf16", tcg.POLICY_GATHER), ("bf16", tcg.POLICY_TILE),
                            ("f16", tcg.POLICY_TILE), ("bf16", tcg.POLICY_AUTO), ("f32", tcg.POLICY_TILE)):
        tcg.sgt_set_policy(meta, policy)
        Y = tcg.spmm(meta, upload_x(X, x_dtype))
        torch.cuda.synchronize()
        assert np.array_equal(Y.cpu().numpy().astype(np.float64), ref), (x_dtype, policy)
    meta.free()


def test_spmm_rectangular_matrix():
    # More columns than rows and the other way round: X has n_cols rows, Y has n_rows rows.
    rng = np.random.default_rng(11)
    for n_rows, n_cols in ((300, 5000), (5000, 300)):
        rows = [rng.choice(n_cols, size=int(rng.integers(0, 60)), replace=False) for _ in range(n_rows)]
        g = csr_from_rows(rows, n_cols)
        X = W.features_normal(n_cols, 64, 2)
        w = rng.standard_normal(g.nnz).astype(np.float32)
        run_spmm_case(g, X, "f32", w, tcg.POLICY_AUTO, TOL_F32)
        run_spmm_case(g, X, "f32", w, tcg.POLICY_TILE, TOL_F32)
        run_spmm_case(g, W.round_to_bf16(X), "bf16", None, tcg.POLICY_TILE, TOL_F32)


@pytest.mark.parametrize("D", [8, 24, 72, 136, 200, 264, 392, 512])
def test_spmm_tile_path_feature_widths(D):
    # Widths that are not a multiple of the 16-column slice, that span two and four feature parts,
    # with and without edge values, padded rows, and outputs that cannot take 16-byte stores.
    c = W.make_config(5, n=64 * 12, d=D, permute=False)
    g, X = c["csr"], c["X"]
    w = np.random.default_rng(D).standard_normal(g.nnz).astype(np.float32)
    run_spmm_case(g, X, "bf16", w, tcg.POLICY_TILE, TOL_MFMA)
    run_spmm_case(g, X.astype(np.float16).astype(np.float32), "f16", None, tcg.POLICY_TILE, TOL_MFMA, pad=8)
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    tcg.sgt_set_policy(meta, tcg.POLICY_TILE)
    Xd = upload_x(X, "bf16")
    ref = oracle.spmm(g.row_ptr, g.col_idx, X, None)
    for y_dtype, tol in ((torch.float32, TOL_F32), (torch.bfloat16, 2.0 ** -8)):
        big = torch.full((g.n_rows, D + 3), float("nan"), dtype=y_dtype, device=dev())
        Y = big[:, 1:D + 1]                                   # odd leading dimension, shifted start
        tcg.spmm(meta, Xd, None, Y=Y)
        torch.cuda.synchronize()
        assert norm_err(Y.to(torch.float32).cpu().numpy(), ref) <= tol
        assert torch.isnan(big[:, 0]).all() and torch.isnan(big[:, D + 1:]).all()   # nothing outside Y
    meta.free()


def test_spmm_tile_path_windows_with_many_edges():
    # Fully dense 16 x 16 blocks: 48 blocks per window give 12,288 edges and 768 condensed columns,
    # beyond what the tile kernel keeps in registers; 2 blocks per window stay inside it.
    for blocks in (2, 48):
        g = W.dense_block_windows(1024, blocks, seed=5)
        X = W.round_to_bf16(W.features_normal(1024, 40, 6))
        w = np.random.default_rng(blocks).standard_normal(g.nnz).astype(np.float32)
        run_spmm_case(g, X, "bf16", None, tcg.POLICY_TILE, TOL_F32)
        run_spmm_case(g, X, "bf16", w, tcg.POLICY_TILE, TOL_MFMA)


@pytest.mark.parametrize("x_dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("D", [1, 3, 10, 20, 50, 100, 150, 250])
def test_rows_that_cannot_be_read_in_16_byte_pieces(x_dtype, D):
    # Widths that are not a multiple of 16 bytes: fp32 rows go element by element, 16-bit rows in pairs
    # when the width is even and element by element when it is odd or the rows start at odd elements.
    c = W.make_config(3, n=2500, d=D)
    g = c["csr"]
    X = c["X"].astype(np.float16).astype(np.float32) if x_dtype == "f16" else W.round_to_bf16(c["X"])
    w = np.random.default_rng(D).standard_normal(g.nnz).astype(np.float32)
    run_spmm_case(g, X, x_dtype, w, tcg.POLICY_AUTO, TOL_F32)
    run_spmm_case(g, X, x_dtype, None, tcg.POLICY_AUTO, TOL_F32, pad=1)       # odd leading dimension
    run_sddmm_case(g, X, x_dtype, tcg.POLICY_AUTO, TOL_F32)
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    big = torch.zeros((g.n_rows, D + 3), dtype=TORCH_DT[x_dtype], device=dev())
    big[:, 1:D + 1] = upload_x(X, x_dtype)
    Xs = big[:, 1:D + 1]                                                       # rows start at an odd element
    out = tcg.sddmm(meta, Xs)
    Y = tcg.spmm(meta, Xs)
    torch.cuda.synchronize()
    assert norm_err(out.cpu().numpy(), oracle.sddmm(g.row_ptr, g.col_idx, X)) <= TOL_F32
    assert norm_err(Y.cpu().numpy(), oracle.spmm(g.row_ptr, g.col_idx, X, None)) <= TOL_F32
    meta.free()


def test_auto_policy_ignores_a_negligible_tile_share():
    # A graph without neighbour sharing in which k windows are replaced by dense 16 x 16 blocks: while these hold
    # less than 2 % of the stored entries the automatic policy sends no window to the tile kernels (a launch
    # over all windows would cost more than it saves); above that it does.  Results are right either way.
    base = W.make_config(5, n=64 * 40, d=8, permute=True)["csr"]
    X = W.round_to_bf16(W.features_normal(base.n_cols, 128, 4))
    for k, expect_tiles in ((1, False), (12, True)):
        rows = [base.col_idx[base.row_ptr[i]:base.row_ptr[i + 1]] for i in range(base.n_rows)]
        for wdw in range(k):
            for r in range(16):
                rows[wdw * 16 + r] = np.arange(100 * wdw, 100 * wdw + 16, dtype=np.int32)
        g = csr_from_rows(rows, base.n_cols)
        assert (256 * k * 50 < g.nnz) == (not expect_tiles)
        st = run_spmm_case(g, X, "bf16", None, tcg.POLICY_AUTO, TOL_F32)
        assert (st["n_tile_windows"] >= k) if expect_tiles else (st["n_tile_windows"] == 0 and st["nnz_tile"] == 0)
        run_sddmm_case(g, X, "bf16", tcg.POLICY_AUTO, TOL_F32)
        st = run_spmm_case(g, X, "bf16", None, tcg.POLICY_TILE, TOL_F32)
        assert st["nnz_tile"] == g.nnz                              # a forced policy is taken literally


@pytest.mark.parametrize("D", [24, 72, 136, 264])
def test_spmm_tile_path_with_32_row_windows(D):
    # Windows of 32 rows: two MFMA row blocks per wavefront.  Clustered graph (windows share neighbours),
    # forced and automatic policy, with and without edge values, ragged last window, bf16 output.
    c = W.make_config(5, n=64 * 12, d=D, permute=False)
    full, X = c["csr"], c["X"]
    n_keep = 64 * 12 - 23                                       # last window has 9 rows
    g = CSR(n_keep, full.n_cols, full.row_ptr[:n_keep + 1].copy(), full.col_idx[:full.row_ptr[n_keep]].copy())
    w = np.random.default_rng(D).standard_normal(g.nnz).astype(np.float32)
    for policy in (tcg.POLICY_TILE, tcg.POLICY_AUTO):
        st = run_spmm_case(g, X, "bf16", w, policy, TOL_MFMA, H=32)
        if policy == tcg.POLICY_TILE or D >= 64:
            assert st["n_tile_windows"] > 0
        run_spmm_case(g, X, "bf16", None, policy, TOL_F32, H=32)
    run_spmm_case(g, X.astype(np.float16).astype(np.float32), "f16", None, tcg.POLICY_TILE, TOL_MFMA, H=32, pad=8)
    run_spmm_case(g, X, "bf16", None, tcg.POLICY_TILE, 2.0 ** -8, H=32, y_dtype=torch.bfloat16)
    run_sddmm_case(g, W.round_to_bf16(X), "bf16", tcg.POLICY_TILE, TOL_F32, H=32)      # SDDMM keeps to the gather path here
    # a window with more edges than fit in registers under a forced policy, and a hub window
    gd = W.dense_block_windows(1024, 5, seed=9)
    Xd = W.round_to_bf16(W.features_normal(1024, D, 7))
    run_spmm_case(gd, Xd, "bf16", None, tcg.POLICY_TILE, TOL_F32, H=32)
    run_spmm_case(gd, Xd, "bf16", None, tcg.POLICY_AUTO, TOL_F32, H=32)


def test_spmm_bf16_output():
    c = W.make_config(5, n=64 * 20, d=64, permute=False)
    for policy in (tcg.POLICY_GATHER, tcg.POLICY_TILE):
        run_spmm_case(c["csr"], c["X"], "bf16", None, policy, 2.0 ** -8, y_dtype=torch.bfloat16)


@pytest.mark.parametrize("x_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("y_dtype", [torch.bfloat16, torch.float16])
def test_spmm_gather_sixteen_bit_output(x_dtype, y_dtype):
    """Rows with and without split segments (hubs of an R-MAT graph) written as 16-bit values: packed stores
    when the output rows are 8-byte aligned, scalar ones for a view that starts one element later."""
    c = W.make_config(4, n=6000, d=64)
    g = c["csr"]
    X = W.round_to_bf16(c["X"]) if x_dtype == "bf16" else c["X"]
    tol = 2.0 ** -8 if y_dtype == torch.bfloat16 else 2.0 ** -10
    stats = run_spmm_case(g, X, x_dtype, None, tcg.POLICY_GATHER, tol, y_dtype=y_dtype)
    assert stats["n_long_rows"] > 0
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    tcg.sgt_set_policy(meta, tcg.POLICY_GATHER)
    big = torch.full((g.n_rows, 64 + 4), float("nan"), dtype=y_dtype, device=dev())
    Y = big[:, 1:65]                                       # rows start 2 bytes off an 8-byte boundary
    tcg.spmm(meta, upload_x(X, x_dtype), None, Y=Y)
    torch.cuda.synchronize()
    meta.free()
    ref = oracle.spmm(g.row_ptr, g.col_idx, X, None)
    assert norm_err(Y.to(torch.float32).cpu().numpy(), ref) <= tol
    assert torch.isnan(big[:, 0]).all() and torch.isnan(big[:, 65:]).all()


def test_spmm_is_deterministic():
    c = W.make_config(4, n=20000, d=64)
    rp, ci = upload_csr(c["csr"])
    meta = tcg.sgt_build(rp, ci, 16, 8)
    Xd = upload_x(c["X"], "f32")
    Y1 = tcg.spmm(meta, Xd).clone()
    Y2 = tcg.spmm(meta, Xd)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y2)
    meta.free()


# ----------------------------------------------------------------------------------------------
# SDDMM and row softmax
# ----------------------------------------------------------------------------------------------

def run_sddmm_case(g, X, x_dtype, policy, tol, H=16):
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, H, 16, n_cols=g.n_cols)
    tcg.sgt_set_policy(meta, policy)
    out = torch.full((g.nnz,), float("nan"), device=dev())
    tcg.sddmm(meta, upload_x(X, x_dtype), out=out)
    torch.cuda.synchronize()
    err = norm_err(out.cpu().numpy(), oracle.sddmm(g.row_ptr, g.col_idx, X))
    meta.free()
    assert err <= tol, "normalised error %.3g above %.1g" % (err, tol)


@pytest.mark.parametrize("cfg,n,D", [(3, 20000, 32), (1, 2048, 16), (2, 5000, 64), (4, 8000, 128),
                                     (3, 3000, 5), (3, 3000, 48), (4, 2000, 320), (3, 1000, 1100)])
def test_sddmm_fp32(cfg, n, D):
    c = W.make_config(cfg, n=n, d=D)
    run_sddmm_case(c["csr"], c["X"], "f32", tcg.POLICY_AUTO, TOL_F32)


def test_sddmm_hub_rows():
    g = hub_graph()
    run_sddmm_case(g, W.features_normal(g.n_cols, 32, 1), "f32", tcg.POLICY_AUTO, TOL_F32)


@pytest.mark.parametrize("x_dtype", ["bf16", "f16"])
@pytest.mark.parametrize("policy", [tcg.POLICY_GATHER, tcg.POLICY_TILE, tcg.POLICY_AUTO])
def test_sddmm_16bit_features(x_dtype, policy):
    rnd = W.round_to_bf16 if x_dtype == "bf16" else (lambda a: a.astype(np.float16).astype(np.float32))
    for cfg, n, D, permute in ((5, 64 * 60, 256, False), (5, 64 * 30, 64, True), (3, 4000, 32, True),
                               (5, 64 * 10, 72, False), (4, 3000, 512, True)):
        c = W.make_config(cfg, n=n, d=D, permute=permute)
        run_sddmm_case(c["csr"], rnd(c["X"]), x_dtype, policy, TOL_F32)   # exact products, fp32 sums on both paths


@pytest.mark.parametrize("policy", [tcg.POLICY_TILE, tcg.POLICY_AUTO])
def test_sddmm_fp32_features_on_the_tile_path(policy):
    # fp32 operands split exactly into bf16 triples, six MFMAs per K step: the fp32 tolerance applies.  Widths
    # with a ragged last K step, windows of both classes (<= 512 edges / more), rows beyond the last window.
    for cfg, n, D, permute in ((5, 64 * 60, 256, False), (5, 64 * 30, 64, True), (3, 4000, 32, True),
                               (5, 64 * 10, 72, False), (4, 3000, 128, True), (5, 64 * 12, 200, False),
                               (5, 64 * 12 , 4, False)):
        c = W.make_config(cfg, n=n, d=D, permute=permute)
        run_sddmm_case(c["csr"], c["X"], "f32", policy, TOL_F32)
    for blocks, D in ((2, 40), (20, 136), (48, 40)):
        g = W.dense_block_windows(1024, blocks, seed=5)
        run_sddmm_case(g, W.features_normal(1024, D, 6), "f32", policy, TOL_F32)
    g = hub_graph(1000)
    run_sddmm_case(g, W.features_normal(g.n_cols, 96, 1), "f32", policy, TOL_F32)


def test_sddmm_fp32_tile_path_is_as_accurate_as_fp32_arithmetic():
    # As for SpMM: every score must be within fp32 rounding of sum |x_i||x_j| over the features, also when the
    # magnitudes of the features differ by many binades (a wrong or missing term of the split is 2^-16 of a
    # product).  The gather path is held to the same bound.
    c = W.make_config(5, n=64 * 60, d=256, permute=False)
    g = c["csr"]
    rng = np.random.default_rng(2)
    X = (rng.standard_normal((g.n_cols, 256)) * np.exp2(rng.integers(-12, 13, (g.n_cols, 256)))).astype(np.float32)
    ref = oracle.sddmm(g.row_ptr, g.col_idx, X)
    mag = oracle.sddmm(g.row_ptr, g.col_idx, np.abs(X))
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    for policy in (tcg.POLICY_GATHER, tcg.POLICY_TILE):
        tcg.sgt_set_policy(meta, policy)
        out = tcg.sddmm(meta, upload_x(X, "f32"))
        torch.cuda.synchronize()
        rel = np.abs(out.cpu().numpy().astype(np.float64) - ref) / np.maximum(mag, 1e-300)
        assert rel.max() <= 2.0 ** -19, (policy, rel.max())
    meta.free()


def test_sddmm_integer_and_one_hot_inputs_are_exact():
    g = hub_graph(2000)
    rng = np.random.default_rng(0)
    X = rng.integers(-4, 5, (g.n_cols, 64)).astype(np.float32)
    ref = oracle.sddmm(g.row_ptr, g.col_idx, X)
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 16)
    for x_dtype, policy in (("f32", tcg.POLICY_GATHER), ("bf16", tcg.POLICY_GATHER), ("bf16", tcg.POLICY_TILE),
                            ("f16", tcg.POLICY_TILE), ("f32", tcg.POLICY_TILE)):
        tcg.sgt_set_policy(meta, policy)
        out = tcg.sddmm(meta, upload_x(X, x_dtype))
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().astype(np.float64), ref), (x_dtype, policy)
    meta.free()


def test_row_softmax_and_attention_chain():
    c = W.make_config(3, n=20000)
    g, X = c["csr"], c["X"]
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    Xd = upload_x(X, "f32")
    e = tcg.sddmm(meta, Xd)
    p = tcg.row_softmax(meta, e)
    Y = tcg.spmm(meta, Xd, p)
    torch.cuda.synchronize()
    e_ref = oracle.sddmm(g.row_ptr, g.col_idx, X)
    assert norm_err(e.cpu().numpy(), e_ref) <= TOL_F32
    # softmax is checked on the library's own SDDMM output (its input), then the chain end to end
    p_ref_own = oracle.row_softmax(g.row_ptr, e.cpu().numpy().astype(np.float64))
    assert norm_err(p.cpu().numpy(), p_ref_own) <= TOL_F32
    p_ref = oracle.row_softmax(g.row_ptr, e_ref)
    Y_ref = oracle.spmm(g.row_ptr, g.col_idx, X, p_ref.astype(np.float32))
    assert norm_err(Y.cpu().numpy(), Y_ref) <= 1e-4      # exp() amplifies the fp32 rounding of e by |e|
    q = tcg.row_softmax(meta, e, out=e)                  # in place
    torch.cuda.synchronize()
    assert torch.equal(q, p)
    meta.free()


def test_row_softmax_and_its_gradient_at_every_row_length_class():
    # Row lengths on both sides of every switch between kernels and variants (lane groups of 4, 8 and 16 up to 128
    # entries, one wavefront with the row in registers up to 512, 1,024 and 2,048, pieces of 4,096 entries spread
    # over workgroups beyond), empty rows in between, scores large enough that an unshifted exp would overflow.
    lengths = [0, 1, 2, 15, 16, 17, 31, 33, 64, 127, 128, 129, 130, 255, 256, 257, 511, 512, 513, 1000, 1024, 1025,
               2047, 2048, 2049, 2050, 4095, 4096, 4097, 8191, 8192, 8193, 9000, 0, 3, 0, 5, 7, 8, 9, 12, 24, 32, 40,
               20000]
    n_cols = 20001
    rng = np.random.default_rng(21)
    g = csr_from_rows([np.sort(rng.choice(n_cols, size=k, replace=False)) for k in lengths], n_cols)
    v = (rng.standard_normal(g.nnz) * 30.0 + 80.0).astype(np.float32)
    dp = rng.standard_normal(g.nnz).astype(np.float32)
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8, n_cols=n_cols)
    p = tcg.row_softmax(meta, torch.from_numpy(v).to(dev()))
    dv = tcg.row_softmax_backward(meta, p, torch.from_numpy(dp).to(dev()))
    torch.cuda.synchronize()
    p_ref = oracle.row_softmax(g.row_ptr, v.astype(np.float64))
    assert np.isfinite(p.cpu().numpy()).all()
    assert norm_err(p.cpu().numpy(), p_ref) <= TOL_F32
    sums = np.add.reduceat(p.cpu().numpy().astype(np.float64), g.row_ptr[:-1][np.diff(g.row_ptr) > 0])
    np.testing.assert_allclose(sums, 1.0, atol=1e-5)
    dv_ref = oracle.row_softmax_backward(g.row_ptr, p.cpu().numpy().astype(np.float64), dp.astype(np.float64))
    assert norm_err(dv.cpu().numpy(), dv_ref) <= TOL_F32
    # in place, and a very long row one of whose pieces holds nothing but -inf (masked scores): zeros there
    v2 = v.copy()
    b = int(g.row_ptr[len(lengths) - 1])
    v2[b + 4096:b + 8192] = -np.inf
    q = torch.from_numpy(v2).to(dev())
    q2 = tcg.row_softmax(meta, q, out=q)
    torch.cuda.synchronize()
    q_ref = oracle.row_softmax(g.row_ptr, v2.astype(np.float64))
    assert np.isfinite(q2.cpu().numpy()).all() and (q2.cpu().numpy()[b + 4096:b + 8192] == 0).all()
    assert norm_err(q2.cpu().numpy(), q_ref) <= TOL_F32
    d2 = torch.from_numpy(dp).to(dev())
    d2 = tcg.row_softmax_backward(meta, p, d2, out=d2)
    torch.cuda.synchronize()
    assert torch.equal(d2, dv)
    meta.free()
    # graphs whose rows all stay below 8, 16 and 32 entries: the variants with 4, 8 and 16 lanes per row
    for cap in (8, 16, 32):
        g = csr_from_rows([np.sort(rng.choice(500, size=int(k), replace=False)) for k in rng.integers(0, cap + 1, 300)], 500)
        v = (rng.standard_normal(g.nnz) * 30.0 + 80.0).astype(np.float32)
        dp = rng.standard_normal(g.nnz).astype(np.float32)
        rp, ci = upload_csr(g)
        meta = tcg.sgt_build(rp, ci, 16, 8, n_cols=500)
        p = tcg.row_softmax(meta, torch.from_numpy(v).to(dev()))
        dv = tcg.row_softmax_backward(meta, p, torch.from_numpy(dp).to(dev()))
        torch.cuda.synchronize()
        assert norm_err(p.cpu().numpy(), oracle.row_softmax(g.row_ptr, v.astype(np.float64))) <= TOL_F32, cap
        dv_ref = oracle.row_softmax_backward(g.row_ptr, p.cpu().numpy().astype(np.float64), dp.astype(np.float64))
        assert norm_err(dv.cpu().numpy(), dv_ref) <= TOL_F32, cap
        meta.free()


def test_attention_chain_replays_from_a_hip_graph():
    # SDDMM -> row softmax -> SpMM (and the fused call) captured once into a HIP graph and replayed with fresh
    # inputs: after the first eager call has sized the library's scratch, the calls neither allocate nor
    # synchronise, so a launch-bound layer can be replayed as one graph launch.  Every replay is checked
    # against the eager result bit for bit, with eager work and synchronisations between the replays.
    c = W.make_config(3, n=20000)
    g = c["csr"]
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, 16, 8)
    rng = np.random.default_rng(8)
    inputs = [torch.from_numpy(rng.standard_normal(c["X"].shape).astype(np.float32)).to(dev()) for _ in range(3)]
    Xs = inputs[0].clone()
    e = torch.empty(g.nnz, device=dev())
    p = torch.empty(g.nnz, device=dev())
    Y = torch.empty_like(Xs)
    Yf = torch.empty_like(Xs)

    def chain():
        tcg.sddmm(meta, Xs, out=e)
        tcg.row_softmax(meta, e, out=p)
        tcg.spmm(meta, Xs, p, Y=Y)
        tcg.attention(meta, Xs, Y=Yf)

    eager = []
    for X in inputs:                                         # eager reference (also sizes the scratch buffers)
        Xs.copy_(X)
        chain()
        torch.cuda.synchronize()
        eager.append((Y.clone(), Yf.clone(), p.clone()))
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            chain()
    torch.cuda.synchronize()
    for rnd in range(2):
        for X, (Y_ref, Yf_ref, p_ref) in zip(inputs, eager):
            Xs.copy_(X)
            Y.fill_(float("nan"))
            Yf.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(Y, Y_ref) and torch.equal(Yf, Yf_ref) and torch.equal(p, p_ref), rnd
            tcg.spmm(meta, X)                                # unrelated eager work between the replays
            torch.cuda.synchronize()
    meta.free()


def test_reserved_scratch_lets_wide_features_be_captured_without_a_warm_up():
    # The plan reserves partial-sum scratch for D <= 128.  A wider first call regrows it, which a stream under
    # capture cannot do: the call then reports TCG_ESCRATCH and leaves the capture intact; after
    # tcg_sgt_reserve the same call is captured and replays to the oracle's result.
    import ctypes
    g = hub_graph(2500, seed=9)
    rp, ci = upload_csr(g)
    D = 256
    X = W.features_uniform(g.n_cols, D, 4)
    Xd = upload_x(X, "f32")
    Y = torch.empty((g.n_rows, D), device=dev())
    Y_ref = oracle.spmm(g.row_ptr, g.col_idx, X, None)
    lib = tcg.load_library()
    for reserve_first in (False, True):
        meta = tcg.sgt_build(rp, ci, 16, 8)
        assert tcg.sgt_plan_stats(meta)["n_long_rows"] > 0
        if reserve_first:
            tcg.sgt_reserve(meta, D)
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        status = None
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                status = lib.tcg_spmm(meta._h, ctypes.c_void_p(Xd.data_ptr()), 0, D, D, None,
                                      ctypes.c_void_p(Y.data_ptr()), 0, D, ctypes.c_void_p(side.cuda_stream))
                Xd.add_(0.0)                                   # the capture is still alive after a refusal
        torch.cuda.synchronize()
        if not reserve_first:
            assert status == -6 and b"tcg_sgt_reserve" in lib.tcg_strerror(status)
        else:
            assert status == 0
            for _ in range(2):
                Y.fill_(float("nan"))
                graph.replay()
                torch.cuda.synchronize()
                assert norm_err(Y.cpu().numpy(), Y_ref) <= TOL_F32
                tcg.sddmm(meta, Xd)                            # eager work between the replays
                torch.cuda.synchronize()
        del graph
        meta.free()


@pytest.mark.parametrize("x_dtype", ["f32", "bf16"])
def test_non_finite_features_reach_the_rows_the_header_says(x_dtype):
    # One infinite feature row X[j].  Gather path: exactly the rows with an entry in column j become
    # non-finite (Equation 1 applied to the stored entries).  Condensed-tile path: every row of every
    # window whose column list contains j (0 x inf inside the matrix unit); all other rows stay exact.
    c = W.make_config(5, n=64 * 30, d=128, permute=False)
    g = c["csr"]
    X = W.round_to_bf16(c["X"]) if x_dtype == "bf16" else c["X"].copy()
    j = 777
    X[j, :] = np.inf
    rp, ci = upload_csr(g)
    Xd = torch.from_numpy(X).to(dev()).to(TORCH_DT[x_dtype])
    rows_with_j = np.zeros(g.n_rows, dtype=bool)
    for i in range(g.n_rows):
        rows_with_j[i] = j in g.col_idx[g.row_ptr[i]:g.row_ptr[i + 1]]
    win_with_j = rows_with_j.reshape(-1, 16).any(axis=1).repeat(16)
    Xz = X.copy()
    Xz[j, :] = 0.0
    Y_clean = oracle.spmm(g.row_ptr, g.col_idx, Xz, None)
    for policy, bad in ((tcg.POLICY_GATHER, rows_with_j), (tcg.POLICY_TILE, win_with_j)):
        meta = tcg.sgt_build(rp, ci, 16, 8)
        tcg.sgt_set_policy(meta, policy)
        Y = tcg.spmm(meta, Xd).cpu().numpy()
        finite = np.isfinite(Y).all(axis=1)
        assert np.array_equal(~finite, bad), policy
        tol = TOL_F32 if (x_dtype == "f32" or policy == tcg.POLICY_GATHER) else TOL_MFMA
        assert norm_err(Y[finite], Y_clean[finite]) <= tol
        meta.free()


def test_calls_follow_the_current_stream():
    # The binding passes torch's current stream: the whole path on a side stream must give the same bits
    # as on the default stream, and the work must really be enqueued there (the side stream's event
    # completes only after the library's kernels).
    c = W.make_config(4, n=30000, d=64)
    g, X = c["csr"], c["X"]
    rp, ci = upload_csr(g)
    Xd = upload_x(X, "f32")
    meta0 = tcg.sgt_build(rp, ci, 16, 8)
    Y0 = tcg.spmm(meta0, Xd)
    e0 = tcg.sddmm(meta0, Xd)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        meta1 = tcg.sgt_build(rp, ci, 16, 8)
        Y1 = tcg.spmm(meta1, Xd)
        e1 = tcg.sddmm(meta1, Xd)
        p1 = tcg.row_softmax(meta1, e1)
        done = torch.cuda.Event()
        done.record(side)
    done.synchronize()
    assert torch.equal(Y0, Y1) and torch.equal(e0, e1)
    assert np.array_equal(tcg.sgt_export(meta0)["edge_to_col"].cpu().numpy(), tcg.sgt_export(meta1)["edge_to_col"].cpu().numpy())
    S = oracle.row_softmax(g.row_ptr, e1.cpu().numpy().astype(np.float64))
    assert norm_err(p1.cpu().numpy(), S) <= TOL_F32
    meta0.free()
    meta1.free()


def _random_graph(rng):
    """Graphs nobody would draw on purpose: random shape, a random mix of empty rows, short rows, hub rows, rows
    of one window sharing a column set, sorted or shuffled column order, column spaces from tiny to beyond the
    LDS bitmap."""
    n_rows = int(rng.integers(1, 6000))
    n_cols = int(rng.choice([rng.integers(1, 3000), rng.integers(3000, 150000), rng.integers(1200000, 2500000)]))
    kind = int(rng.integers(0, 4))
    shared = np.sort(rng.choice(n_cols, size=min(n_cols, int(rng.integers(1, 500))), replace=False))
    lens = np.where(rng.random(n_rows) < 0.3, 0, rng.integers(1, 30, n_rows))
    for _ in range(int(rng.integers(0, 5))):
        lens[rng.integers(0, n_rows)] = int(rng.integers(150, 9000)) if rng.random() < 0.8 else int(rng.integers(9000, 60000))
    rows = []
    for i in range(n_rows):
        k = min(int(lens[i]), n_cols)
        if k == 0:
            rows.append(np.zeros(0, np.int32))
            continue
        if kind == 1 or (kind == 2 and (i // 16) % 2 == 0):
            cols = rng.choice(shared, size=min(k, len(shared)), replace=False)
        elif kind == 3 and (i // 16) % 5 == 0:
            cols = shared
        else:
            cols = rng.choice(n_cols, size=k, replace=False) if k * 4 < n_cols else rng.permutation(n_cols)[:k]
        cols = np.asarray(cols, dtype=np.int32)
        rows.append(np.sort(cols) if rng.random() < 0.7 else cols)
    return csr_from_rows(rows, n_cols)


@pytest.mark.parametrize("seed", range(12))
def test_random_graphs_every_operation_against_the_oracle(seed):
    rng = np.random.default_rng(1000 + seed)
    g = _random_graph(rng)
    D = int(rng.choice([4, 16, 32, 64, 72, 128, 200, 256]))
    if max(g.n_rows, g.n_cols) * D > 1.5e8:
        D = 16
    x_dtype = str(rng.choice(["f32", "bf16", "f16"]))
    H = int(rng.choice([16, 16, 32, 7]))
    policy = [tcg.POLICY_AUTO, tcg.POLICY_GATHER, tcg.POLICY_TILE][int(rng.integers(0, 3))]
    if H == 7:
        policy = tcg.POLICY_AUTO
    weighted = bool(rng.random() < 0.5)
    case = dict(seed=seed, n_rows=g.n_rows, n_cols=g.n_cols, nnz=g.nnz, D=D, x=x_dtype, H=H, policy=int(policy), w=weighted)
    X = W.features_normal(max(g.n_rows, g.n_cols), D, seed)
    X = W.round_to_bf16(X) if x_dtype == "bf16" else (X.astype(np.float16).astype(np.float32) if x_dtype == "f16" else X)
    w = rng.standard_normal(g.nnz).astype(np.float32) if weighted else None
    rp, ci = upload_csr(g)
    meta = tcg.sgt_build(rp, ci, H, 8, n_cols=g.n_cols)
    check_sgt(meta, g, H, 8)
    tcg.sgt_set_policy(meta, policy)
    Xd = upload_x(X, x_dtype)
    tile_possible = policy != tcg.POLICY_GATHER and x_dtype != "f32"
    Y = torch.full((g.n_rows, D), float("nan"), device=dev())
    tcg.spmm(meta, Xd, None if w is None else torch.from_numpy(w).to(dev()), Y=Y)
    torch.cuda.synchronize()
    err = norm_err(Y.cpu().numpy(), oracle.spmm(g.row_ptr, g.col_idx, X[:g.n_cols], w))
    assert err <= (TOL_MFMA if (weighted and tile_possible) else TOL_F32), ("spmm", err, case)
    if g.nnz:
        e = torch.full((g.nnz,), float("nan"), device=dev())
        tcg.sddmm(meta, Xd, out=e)
        torch.cuda.synchronize()
        err = norm_err(e.cpu().numpy(), oracle.sddmm(g.row_ptr, g.col_idx, X))
        assert err <= TOL_F32, ("sddmm", err, case)
        v = (rng.standard_normal(g.nnz) * 10).astype(np.float32)
        p = tcg.row_softmax(meta, torch.from_numpy(v).to(dev()))
        dp = rng.standard_normal(g.nnz).astype(np.float32)
        dv = tcg.row_softmax_backward(meta, p, torch.from_numpy(dp).to(dev()))
        torch.cuda.synchronize()
        assert norm_err(p.cpu().numpy(), oracle.row_softmax(g.row_ptr, v.astype(np.float64))) <= TOL_F32, ("softmax", case)
        dv_ref = oracle.row_softmax_backward(g.row_ptr, p.cpu().numpy().astype(np.float64), dp.astype(np.float64))
        assert norm_err(dv.cpu().numpy(), dv_ref) <= TOL_F32, ("softmax gradient", case)
    meta.free()
