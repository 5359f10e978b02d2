"""GPU parity of marlaas_lora_fwd_multi (several projections of one input in one call, through
the C ABI) against the fp64 oracle applied to each projection, plus its error paths.  Tolerance as
for the single-projection forward: floored relative error max <= 1e-2, mean <= 1e-3, fp32 outputs."""
import numpy as np
import pytest
import torch

from paper_2605_08527_amd import api
from harness import workloads as wl
from helpers import assert_close, to_dev, to_host

pytestmark = pytest.mark.gpu


def _projections(seed, T, K, Ns, ranks_per_proj, scales, ids, layout):
    """One workload per projection, all with the x of the first."""
    ws = [wl.make_layer(seed + 7 * p, T, K, N, list(ranks_per_proj[p]), list(scales), ids, dtype="bf16", layout=layout)
          for p, N in enumerate(Ns)]
    for w in ws[1:]:
        w["x"] = ws[0]["x"]
    return ws


def _run_multi(ws, out_dtype=torch.float32, pad=0):
    ctx = api.marlaas_create(0)
    x = to_dev(ws[0]["x"])
    ids = torch.from_numpy(np.ascontiguousarray(ws[0]["ids"], dtype=np.int32)).cuda()
    n = len(ws[0]["A"])
    seg = api.marlaas_segmap_build(ctx, ids, n)
    keep, descs, ys = [], [], []
    for w in ws:
        W, A, B = to_dev(w["W"]), [to_dev(a) for a in w["A"]], [to_dev(b) for b in w["B"]]
        keep.append((W, A, B))
        d = api.LoraDesc(x, W, A, B, w["ranks"], w["scales"], seg, layout=w["layout"], out_dtype=out_dtype)
        descs.append(d)
        buf = torch.full((x.shape[0], d.shape[2] + pad), float("nan"), dtype=out_dtype, device="cuda")
        ys.append(buf[:, :d.shape[2]])
    nbytes = api.marlaas_workspace_bytes_multi(descs)
    assert nbytes > 0 or x.shape[0] == 0
    wsbuf = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    api.marlaas_set_workspace(ctx, wsbuf)
    api.marlaas_profile_enable(ctx, True)       # counts the GEMM launches: one if the call ran fused
    api.marlaas_lora_fwd_multi(ctx, descs, ys)
    torch.cuda.synchronize()
    launches = api.marlaas_profile_read(ctx, api.MARLAAS_KERNEL_GEMM)[1]
    api.marlaas_profile_enable(ctx, False)
    return ys, (ctx, seg, keep, descs, wsbuf, launches)


def _check(oracle, ws, tag, gemm_launches=None, **kw):
    ys, rest = _run_multi(ws, **kw)
    if gemm_launches is not None:
        assert rest[-1] == gemm_launches, "%s: %d GEMM launches, expected %d" % (tag, rest[-1], gemm_launches)
    for p, (w, y) in enumerate(zip(ws, ys)):
        ref = oracle.fwd(w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"], layout=w["layout"])
        tol = (1e-2, 1e-3) if y.dtype == torch.float32 else (1e-2, 2.5e-3)
        assert_close(to_host(y), ref, "%s projection %d" % (tag, p), *tol)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("ranks", [((8, 16, 24, 32), (16, 16, 8, 8), (32, 8, 16, 24)),
                                   ((1, 5, 12, 16, 7), (3, 3, 3, 3, 3), (16, 4, 2, 9, 40))])
def test_qkv_shaped_small_batch(oracle, layout, ranks):
    """Three projections of unequal width (the second and third not multiples of the 128-wide
    column tile), per-projection ranks, rows without an adapter, a ragged row tile and a contraction
    tail.  The first rank set runs as one GEMM launch in both layouts, the second (ranks that are
    not multiples of 8) only in the contraction-contiguous layout and otherwise one by one."""
    rng = np.random.default_rng(3)
    T, K, Ns = 200, 520, (384, 136, 200)
    n = len(ranks[0])
    ids = rng.integers(-1, n, size=T).astype(np.int32)
    ws = _projections(51, T, K, Ns, ranks, [2.0, 0.5, 1.0, 0.25, 1.5][:n], ids, layout)
    fused = layout == 1 or all(r % 8 == 0 for rr in ranks for r in rr)
    _check(oracle, ws, "qkv", gemm_launches=1 if fused else len(Ns))


@pytest.mark.parametrize("layout", [0, 1])
def test_decode_shaped_two_projections(oracle, layout):
    """gate / up of a decode batch at a size whose concatenated columns span many column tiles and
    several contraction splits: 256 rows, Zipf segment sizes, 16 adapters of rank 16; padded
    outputs, bf16 results."""
    rng = np.random.default_rng(8)
    T, K, Ns, n = 256, 1024, (1536, 1536), 16
    p = 1.0 / np.arange(1, n + 1) ** 1.2
    ids = rng.choice(n, size=T, p=p / p.sum()).astype(np.int32)
    ws = _projections(61, T, K, Ns, [[16] * n] * 2, [2.0] * n, ids, layout)
    _check(oracle, ws, "gate/up", gemm_launches=1, out_dtype=torch.bfloat16, pad=8)


def test_full_size_decode_qkv(oracle):
    """The shape bench.py times for this call: 256 decode tokens (Zipf segment sizes over 32
    adapters of rank 16), d_in 4096, q / k / v of 4096, 1024 and 1024 columns, bf16 outputs, the
    layout bench.py uses; every output element against the oracle."""
    sh, ranks, scales, ids = wl.config_ids(1, 0)
    ws = _projections(101, sh["T"], sh["d_in"], (4096, 1024, 1024), [list(ranks)] * 3, list(scales), ids, wl.TORCH)
    _check(oracle, ws, "decode qkv", gemm_launches=1, out_dtype=torch.bfloat16)


def test_no_adapters_and_single_projection(oracle):
    rng = np.random.default_rng(4)
    T, K = 96, 264
    ids = np.full(T, -1, np.int32)
    ws = _projections(71, T, K, (256, 128), [[], []], [], ids, 1)
    _check(oracle, ws, "base only", gemm_launches=1)
    ids = rng.integers(0, 2, size=T).astype(np.int32)
    ws = _projections(73, T, K, (136,), [[8, 16]], [1.0, 2.0], ids, 0)
    _check(oracle, ws, "single", gemm_launches=1)


def test_ranks_beyond_the_extended_columns_run_projection_by_projection(oracle):
    """640 summed ranks do not fit the 32 extended columns of each of the five column tiles: the
    call runs the projections one after the other through the ordinary kernels, same results."""
    rng = np.random.default_rng(5)
    T, K, n = 300, 328, 3
    ids = rng.integers(-1, n, size=T).astype(np.int32)
    ws = _projections(81, T, K, (264, 136), [[128, 128, 64], [128, 64, 128]], [2.0, 1.0, 0.5], ids, 1)
    _check(oracle, ws, "wide ranks", gemm_launches=2)


def test_mismatched_projections_are_rejected():
    rng = np.random.default_rng(6)
    T, K, n = 64, 128, 2
    ids = rng.integers(0, n, size=T).astype(np.int32)
    ws = _projections(91, T, K, (128, 128), [[8, 8], [8, 8]], [1.0, 1.0], ids, 1)
    ys, (ctx, seg, keep, descs, wsbuf, _) = _run_multi(ws)
    other_x = torch.zeros_like(to_dev(ws[0]["x"]))
    bad = api.LoraDesc(other_x, keep[1][0], keep[1][1], keep[1][2], ws[1]["ranks"], ws[1]["scales"], seg, layout=1,
                       out_dtype=torch.float32)
    assert api.marlaas_workspace_bytes_multi([descs[0], bad]) == 0
    with pytest.raises(api.MarlaasError):
        api.marlaas_lora_fwd_multi(ctx, [descs[0], bad], ys)
    with pytest.raises(api.MarlaasError):
        api.marlaas_lora_fwd_multi(ctx, descs * 5, ys * 5)        # more than MARLAAS_MAX_PROJ


def test_hip_graph_replay_of_the_fused_call():
    """The fused call captured into a HIP graph after one eager call (which fills the table cache)
    and replayed three times with eager work in between: every replay reproduces the eager
    results bit for bit, also after x changed in place."""
    rng = np.random.default_rng(12)
    T, K, n = 160, 512, 4
    ids = rng.integers(-1, n, size=T).astype(np.int32)
    ws = _projections(111, T, K, (384, 128), [[16, 8, 32, 16], [8, 8, 16, 16]], [2.0, 1.0, 0.5, 2.0], ids, wl.TORCH)
    ys, (ctx, seg, keep, descs, wsbuf, launches) = _run_multi(ws)
    assert launches == 1
    x = descs[0].tensors[0]

    def snapshot():
        torch.cuda.synchronize()
        return [y.clone() for y in ys]

    eager = snapshot()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            api.marlaas_lora_fwd_multi(ctx, descs, ys)
    for rep in range(3):
        if rep == 2:
            x.mul_(0.5)
            api.marlaas_lora_fwd_multi(ctx, descs, ys)
            eager = snapshot()
        for y in ys:
            y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(got, eager):
            assert torch.equal(a, b), "replay %d differs from the eager call" % rep
