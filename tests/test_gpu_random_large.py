"""Seeded random large-batch cases through the C ABI against the fp64 oracle: a few thousand rows
against a weight wide enough for the large-batch GEMM (expand by DMA or through registers), the
shrink with both operands by DMA or register-staged (odd ranks of contraction-major factors), the
reductions with equal or very unequal segments (longest first, long ones cut into token chunks),
adapters as lists or in a table, the weight's transposed copy kept or made per call.  Sampled
rows of y and dX and a few adapters' dA / dB at the forward / backward tolerance (floored relative
error max <= 1e-2, mean <= 1e-3, fp32 outputs)."""
import numpy as np
import pytest
import torch

from harness import workloads as wl
from helpers import HipLayer, assert_close, to_host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [1, 7, 23])
def test_random_large_batches(oracle, seed):
    rng = np.random.default_rng(seed)
    for case in range(3):
        T = int(rng.integers(2500, 9000))
        K = 8 * int(rng.integers(32, 160))
        N = 256 * int(rng.integers(6, 14)) + 8 * int(rng.integers(0, 32))
        n = int(rng.choice([1, 3, 8, 40, 200]))
        mult8 = rng.random() < 0.6
        ranks = [int(rng.choice([8, 16, 24, 32, 64, 128] if mult8 else [1, 5, 12, 16, 40, 100])) for _ in range(n)]
        scales = [float(rng.choice([0.25, 0.5, 1.0, 2.0])) for _ in range(n)]
        layout = int(rng.integers(0, 2))
        if rng.random() < 0.5:                       # very unequal segments
            p = 1.0 / np.arange(1, n + 1) ** 1.3
            ids = rng.choice(n, size=T, p=p / p.sum()).astype(np.int32)
        else:
            ids = rng.integers(-1, n, size=T).astype(np.int32)
        if rng.random() < 0.3:
            ids = np.sort(ids)
        table, kept = bool(rng.random() < 0.5), bool(rng.random() < 0.5)
        tag = "seed %d case %d: T=%d K=%d N=%d n=%d mult8=%s layout=%d table=%s kept=%s" % (seed, case, T, K, N, n, mult8, layout, table, kept)
        w = wl.make_layer(5000 + 10 * seed + case, T, K, N, ranks, scales, ids, dtype="bf16", layout=layout, want_dY=True)
        args = (w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"])
        rows = np.unique(rng.integers(0, T, size=160)).astype(np.int64)
        rows_t = torch.from_numpy(rows).cuda()
        sel = sorted(set(int(v) for v in rng.integers(0, n, size=min(n, 4))))
        y_ref = oracle.fwd(*args, layout=layout, rows=rows)
        dX_ref, dA_ref, dB_ref = oracle.bwd(*args, w["dY"], layout=layout, rows=rows, adapters=sel)
        L = HipLayer(w, want_bwd=True, table=table, kept_wt=kept)
        y, u = L.fwd(save_u=True)
        assert bool(torch.isfinite(y).all()), tag
        assert_close(to_host(y[rows_t]), y_ref, tag + " y")
        dX, dA, dB = L.bwd(u_saved=u)
        assert bool(torch.isfinite(dX).all()), tag
        assert_close(to_host(dX[rows_t]), dX_ref, tag + " dX")
        for s_, t in enumerate(sel):
            ga, gb = (dA_ref[s_].T, dB_ref[s_].T) if layout == 1 else (dA_ref[s_], dB_ref[s_])
            assert_close(to_host(dA[t]), ga, tag + " dA[%d]" % t)
            assert_close(to_host(dB[t]), gb, tag + " dB[%d]" % t)
        del L
        torch.cuda.empty_cache()
