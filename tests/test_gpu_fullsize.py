"""GPU parity at the full benchmark sizes (configurations 2, 3, 4), in the launch
configuration bench.py times (torch layout, adapters in a table, prebuilt segment map), seeds 0-2.

Gate: fp32 outputs (the fp32 accumulators as they are) against the fp64 oracle at floored relative
error max <= 1e-2, mean <= 1e-3 per output tensor.  y, dX and u are compared on >= 1024 sampled
rows: both ends of every adapter segment, the rows on either side of row-tile edges of the grouped
order, and seeded random rows; dA_t / dB_t in full, for every adapter of configurations 3 and 4.

Secondary: the same passes with bf16 outputs (what bench.py writes).  The final rounding alone
puts a floor under their error (the oracle's own values rounded to bf16 score about 8.7e-4 mean),
so they are held to that measured floor plus 5 %, and to one bf16 unit in the last place (2^-8) at
the maximum."""
import numpy as np
import pytest
import torch

from paper_2605_08527_amd import api
from harness import workloads as wl
from helpers import HipLayer, assert_close, check_bf16, to_host

pytestmark = pytest.mark.gpu


def _sample_rows(ids, n_extra, seed, tile=256):
    T = ids.shape[0]
    rng = np.random.default_rng(seed)
    order = np.argsort(ids, kind="stable")          # grouped order (ids >= 0 here)
    key = ids[order]
    cuts = np.flatnonzero(np.diff(key))
    first = order[np.r_[0, cuts + 1]]
    last = order[np.r_[cuts, T - 1]]
    edges = np.arange(tile, T, tile)
    edges = edges[rng.permutation(edges.size)[:128]]
    at_edges = order[np.concatenate([edges - 1, edges])] if edges.size else np.zeros(0, np.int64)
    extra = rng.integers(0, T, size=n_extra)
    return np.unique(np.concatenate([first, last, at_edges, extra, [0, T - 1]])).astype(np.int64)


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("cfg,adapters", [(2, None), (3, list(range(16))), (4, list(range(64)))])
def test_full_size(oracle, cfg, adapters, seed):
    w = wl.make_config(cfg, seed=seed, layout=wl.TORCH)
    bwd = w["dY"] is not None
    rows = _sample_rows(w["ids"], 900, 100 * seed + cfg)
    assert rows.size >= 1024
    rows_t = torch.from_numpy(rows).cuda()
    args = (w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"])
    y_ref, u_ref = oracle.fwd(*args, layout=w["layout"], rows=rows, want_u=True)
    if bwd:
        dX_ref, dA_ref, dB_ref = oracle.bwd(*args, w["dY"], layout=w["layout"], rows=rows, adapters=adapters)
    # ---- gate: fp32 outputs
    L = HipLayer(w, out_dtype=torch.float32, want_bwd=bwd, table=True, kept_wt=(seed == 1))
    y, u = L.fwd(save_u=True)
    tag = "cfg%d seed%d" % (cfg, seed)
    assert_close(to_host(y[rows_t]), y_ref, tag + " y")
    assert bool(torch.isfinite(y).all())
    # u_save: s_t (x A_t) in grouped order; grouped position of token i through the exported map
    perm, seg_off = api.marlaas_segmap_export(L.map)
    pos = np.empty(L.T, np.int64)
    pos[perm] = np.arange(L.T)
    sc = np.asarray(w["scales"], np.float64)[w["ids"][rows]]
    want_u = np.zeros((rows.size, u.shape[1]))
    want_u[:, :u_ref.shape[1]] = u_ref * sc[:, None]
    assert_close(to_host(u[torch.from_numpy(pos[rows]).cuda()]), want_u, tag + " u_save")
    del y
    if bwd:
        dX, dA, dB = L.bwd(u_saved=u)
        assert_close(to_host(dX[rows_t]), dX_ref, tag + " dX")
        assert bool(torch.isfinite(dX).all())
        del dX
        for s, t in enumerate(adapters):      # oracle gradients are in math orientation
            assert_close(to_host(dA[t]), dA_ref[s].T, tag + " dA[%d]" % t)
            assert_close(to_host(dB[t]), dB_ref[s].T, tag + " dB[%d]" % t)
        assert all(bool(torch.isfinite(g).all()) for g in dA + dB)
    # ---- secondary: bf16 outputs, same inputs, same map and table
    Lb = HipLayer(w, out_dtype=torch.bfloat16, want_bwd=bwd, table=True)
    del L
    torch.cuda.empty_cache()
    yb, ub = Lb.fwd(save_u=bwd)
    check_bf16(to_host(yb[rows_t]), y_ref, tag + " y")
    if bwd:
        dXb, dAb, dBb = Lb.bwd(u_saved=ub)
        check_bf16(to_host(dXb[rows_t]), dX_ref, tag + " dX")
        for s, t in enumerate(adapters[:4]):
            assert_close(to_host(dAb[t]), dA_ref[s].T, tag + " dA[%d] (bf16-output pass)" % t)
            assert_close(to_host(dBb[t]), dB_ref[s].T, tag + " dB[%d] (bf16-output pass)" % t)


@pytest.mark.parametrize("kept_wt", [False, True], ids=["transpose-per-call", "kept-transpose"])
@pytest.mark.parametrize("layout", [wl.MATH, wl.TORCH])
def test_partial_last_round_of_tiles(oracle, layout, kept_wt):
    """17 x 16 = 272 tiles of 256 x 256: one more than a full round of workgroups, the last row
    tile holding the end of the grouped order (the last adapters and the rows without an
    adapter).  Forward and backward, both layouts (one product of each reads the weight along its
    strided dimension: from a copy transposed into scratch by the call, or from the transposed
    copy the descriptor carries), fp32 outputs, sampled rows."""
    rng = np.random.default_rng(31)
    T, K, N, ranks = 4352, 1024, 4096, [16, 8, 32, 16, 24, 16]
    ids = rng.integers(-1, len(ranks), size=T).astype(np.int32)
    w = wl.make_layer(23, T, K, N, ranks, [2.0, 1.0, 0.5, 2.0, 1.0, 0.5], ids, dtype="bf16", layout=layout, want_dY=True)
    L = HipLayer(w, out_dtype=torch.float32, want_bwd=True, kept_wt=kept_wt)
    if kept_wt:      # the copy is the transpose, bit for bit, and the workspace no longer holds one
        assert torch.equal(L.W_t, L.W.t().contiguous())
        need, without = api.marlaas_workspace_bytes(L.desc, True), api.marlaas_workspace_bytes(HipLayer(w, want_bwd=True).desc, True)
        assert need < without if layout == wl.MATH else need <= without     # (torch layout: this backward is planned with a split contraction)
    rows = _sample_rows(ids, 64, 7)
    rows_t = torch.from_numpy(rows).cuda()
    args = (w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"])
    y, u = L.fwd(save_u=True)
    assert_close(to_host(y[rows_t]), oracle.fwd(*args, layout=layout, rows=rows), "tail y")
    assert bool(torch.isfinite(y).all())
    dX, dA, dB = L.bwd(u_saved=u)
    sel = [0, 5]
    dX_ref, dA_ref, dB_ref = oracle.bwd(*args, w["dY"], layout=layout, rows=rows, adapters=sel)
    assert_close(to_host(dX[rows_t]), dX_ref, "tail dX")
    assert bool(torch.isfinite(dX).all())
    for s, t in enumerate(sel):
        ga, gb = (dA_ref[s].T, dB_ref[s].T) if layout == wl.TORCH else (dA_ref[s], dB_ref[s])
        assert_close(to_host(dA[t]), ga, "tail dA[%d]" % t)
        assert_close(to_host(dB[t]), gb, "tail dB[%d]" % t)


@pytest.mark.parametrize("layout", [wl.MATH, wl.TORCH])
@pytest.mark.parametrize("T", [640, 1536])
def test_mid_size_batches(oracle, layout, T):
    """Between decode and prefill (a few hundred to a few thousand rows against a 2048 x 4096
    weight) the planner weighs 128 x 128 tiles with or without a split contraction against
    256 x 256 tiles with one; at these two sizes the forward and the backward GEMM (whose
    contraction is twice as deep) end up on different ones.  Zipf-sized segments, sampled rows."""
    rng = np.random.default_rng(41)
    K, N, ranks = 2048, 4096, [16] * 12
    p = 1.0 / np.arange(1, len(ranks) + 1) ** 1.2
    ids = rng.choice(len(ranks), size=T, p=p / p.sum()).astype(np.int32)
    w = wl.make_layer(37, T, K, N, ranks, [2.0] * len(ranks), ids, dtype="bf16", layout=layout, want_dY=True)
    L = HipLayer(w, out_dtype=torch.float32, want_bwd=True)
    rows = _sample_rows(ids, 48, 11)
    rows_t = torch.from_numpy(rows).cuda()
    args = (w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"])
    y, u = L.fwd(save_u=True)
    assert_close(to_host(y[rows_t]), oracle.fwd(*args, layout=layout, rows=rows), "mid y")
    assert bool(torch.isfinite(y).all())
    dX, dA, dB = L.bwd(u_saved=u)
    sel = [0, len(ranks) - 1]
    dX_ref, dA_ref, dB_ref = oracle.bwd(*args, w["dY"], layout=layout, rows=rows, adapters=sel)
    assert_close(to_host(dX[rows_t]), dX_ref, "mid dX")
    assert bool(torch.isfinite(dX).all())
    for s, t in enumerate(sel):
        ga, gb = (dA_ref[s].T, dB_ref[s].T) if layout == wl.TORCH else (dA_ref[s], dB_ref[s])
        assert_close(to_host(dA[t]), ga, "mid dA[%d]" % t)
        assert_close(to_host(dB[t]), gb, "mid dB[%d]" % t)


@pytest.mark.parametrize("n_adapters", [150, 400], ids=["12-segments-per-tile", "more-segments-than-the-list-holds"])
@pytest.mark.parametrize("layout", [wl.MATH, wl.TORCH])
def test_many_short_segments_in_a_row_tile(oracle, layout, n_adapters):
    """Large batch whose 256-row tiles each hold many adapter segments (ranks 8 .. 32, multiples of
    8): the expand's extra contraction tiles are listed per row tile and fetched by DMA after the
    main loop; with 400 adapters a row tile has more of them than its list holds and the kernel
    stages the expand through registers instead.  Forward and backward, sampled rows, every tenth
    adapter's gradients."""
    rng = np.random.default_rng(43 + n_adapters)
    T, K, N = 4352, 512, 4096
    ranks = [int(r) for r in rng.choice([8, 16, 24, 32], size=n_adapters)]
    scales = [float(s) for s in rng.choice([2.0, 1.0, 0.5], size=n_adapters)]
    ids = rng.integers(-1, n_adapters, size=T).astype(np.int32)
    w = wl.make_layer(47, T, K, N, ranks, scales, ids, dtype="bf16", layout=layout, want_dY=True)
    L = HipLayer(w, out_dtype=torch.float32, want_bwd=True, table=True, kept_wt=True)
    rows = _sample_rows(ids, 200, 13)
    rows_t = torch.from_numpy(rows).cuda()
    args = (w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"])
    y, u = L.fwd(save_u=True)
    assert_close(to_host(y[rows_t]), oracle.fwd(*args, layout=layout, rows=rows), "y")
    assert bool(torch.isfinite(y).all())
    dX, dA, dB = L.bwd(u_saved=u)
    sel = list(range(0, n_adapters, 10))
    dX_ref, dA_ref, dB_ref = oracle.bwd(*args, w["dY"], layout=layout, rows=rows, adapters=sel)
    assert_close(to_host(dX[rows_t]), dX_ref, "dX")
    assert bool(torch.isfinite(dX).all())
    for s, t in enumerate(sel):
        ga, gb = (dA_ref[s].T, dB_ref[s].T) if layout == wl.TORCH else (dA_ref[s], dB_ref[s])
        assert_close(to_host(dA[t]), ga, "dA[%d]" % t)
        assert_close(to_host(dB[t]), gb, "dB[%d]" % t)
