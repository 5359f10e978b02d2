"""GPU parity at the full benchmark sizes (configurations 2, 3, 4), in the launch
configuration bench.py times (torch layout, bf16 outputs, prebuilt segment map):
y and dX are compared with the oracle on a seeded sample of rows that includes
both ends of every adapter segment, dA_t / dB_t in full for a sample of
adapters.  Tolerance: the bf16-output bounds (max 1e-2, mean 2.5e-3: the final
rounding alone costs about 1.4e-3 mean) for y / dX, 1e-2 / 1e-3 for the fp32
gradients."""
import numpy as np
import pytest
import torch

from harness import workloads as wl
from helpers import HipLayer, assert_close, to_host

pytestmark = pytest.mark.gpu


def _sample_rows(ids, n_extra, seed):
    T = ids.shape[0]
    rng = np.random.default_rng(seed)
    order = np.argsort(ids, kind="stable")
    key = ids[order]
    first = order[np.r_[0, np.flatnonzero(np.diff(key)) + 1]]
    last = order[np.r_[np.flatnonzero(np.diff(key)), T - 1]]
    extra = rng.integers(0, T, size=n_extra)
    return np.unique(np.concatenate([first, last, extra, [0, T - 1]])).astype(np.int64)


@pytest.mark.parametrize("cfg,n_extra,adapters", [(2, 96, None), (3, 48, [0, 15]), (4, 96, [0, 7, 21, 40, 63])])
def test_full_size_sampled(oracle, cfg, n_extra, adapters):
    w = wl.make_config(cfg, seed=0, layout=wl.TORCH)
    bwd = w["dY"] is not None
    L = HipLayer(w, out_dtype=torch.bfloat16, want_bwd=bwd)
    rows = _sample_rows(w["ids"], n_extra, 100 + cfg)
    args = (w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"])
    y, u = L.fwd(save_u=bwd)
    y_ref = oracle.fwd(*args, layout=w["layout"], rows=rows)
    rows_t = torch.from_numpy(rows).cuda()
    assert_close(to_host(y[rows_t]), y_ref, "cfg%d y" % cfg, 1e-2, 2.5e-3)
    assert bool(torch.isfinite(y.float()).all())
    if bwd:
        dX, dA, dB = L.bwd(u_saved=u)
        dX_ref, dA_ref, dB_ref = oracle.bwd(*args, w["dY"], layout=w["layout"], rows=rows, adapters=adapters)
        assert_close(to_host(dX[rows_t]), dX_ref, "cfg%d dX" % cfg, 1e-2, 2.5e-3)
        for s, t in enumerate(adapters):      # oracle gradients are in math orientation
            assert_close(to_host(dA[t]), dA_ref[s].T, "cfg%d dA[%d]" % (cfg, t))
            assert_close(to_host(dB[t]), dB_ref[s].T, "cfg%d dB[%d]" % (cfg, t))
        assert all(bool(torch.isfinite(g).all()) for g in dA + dB)


@pytest.mark.parametrize("layout", [wl.MATH, wl.TORCH])
def test_partial_last_round_of_tiles(oracle, layout):
    """17 x 16 = 272 tiles of 256 x 256: one more than a full round of workgroups, the last row
    tile holding the end of the grouped order (the last adapters and the rows without an
    adapter).  Forward and backward, both layouts (one of which transposes the weight into
    scratch at this size), fp32 outputs, sampled rows."""
    rng = np.random.default_rng(31)
    T, K, N, ranks = 4352, 1024, 4096, [16, 8, 32, 16, 24, 16]
    ids = rng.integers(-1, len(ranks), size=T).astype(np.int32)
    w = wl.make_layer(23, T, K, N, ranks, [2.0, 1.0, 0.5, 2.0, 1.0, 0.5], ids, dtype="bf16", layout=layout, want_dY=True)
    L = HipLayer(w, out_dtype=torch.float32, want_bwd=True)
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
