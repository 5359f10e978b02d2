"""GPU parity: the HIP library (through the C ABI) against the fp64 oracle,
element by element, on the same seeded inputs.  Tolerance: floored relative
error max <= 1e-2 and mean <= 1e-3 per output tensor (bf16 inputs, fp32
accumulation); fp32 outputs of the fp32 path are held to 1e-4 / 1e-5."""
import numpy as np
import pytest
import torch

from paper_2605_08527_amd import api
from harness import workloads as wl
from helpers import HipLayer, assert_close, oracle_grads_in_layout, to_host

pytestmark = pytest.mark.gpu


def _oracle_all(oracle, w, bwd):
    args = (w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"])
    y = oracle.fwd(*args, layout=w["layout"])
    if not bwd:
        return y, None, None, None
    dX, dA, dB = oracle.bwd(*args, w["dY"], layout=w["layout"])
    dA, dB = oracle_grads_in_layout(dA, dB, w["layout"])
    return y, dX, dA, dB


@pytest.fixture(params=["lists", "table", "table+packed", "lists+packed", "table+in-kernel+packed", "table+generic+packed"])
def use_table(request, monkeypatch):
    """Adapters given as host pointer lists in the descriptor, or registered in an adapter table object;
    with or without packed copies of the weight (which small batches then read); and, with packed
    copies, the other two ways of finishing the decode kernel's call: by the kernel itself and by
    the generic finish kernel (MARLAAS_DECODE_FINISH=1 / 0, read when the context is created)."""
    if "in-kernel" in request.param:
        monkeypatch.setenv("MARLAAS_DECODE_FINISH", "1")
    if "generic" in request.param:
        monkeypatch.setenv("MARLAAS_DECODE_FINISH", "0")
    return request.param


def check_u_save(oracle, w, L, u, tag=""):
    """u_save holds s_t (x A_t) per token in the grouped order of the map: compare with the
    oracle's u, rows taken through the exported permutation; the padding ranks must be zero."""
    if L.n == 0 or u is None:
        return
    args = (w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"])
    _, u_ref = oracle.fwd(*args, layout=w["layout"], want_u=True)
    perm, seg_off = api.marlaas_segmap_export(L.map)
    T_lora = int(seg_off[L.n])
    if T_lora == 0:
        return
    toks = perm[:T_lora]
    ranks = np.asarray(w["ranks"])[w["ids"][toks]]
    want = np.zeros((T_lora, u.shape[1]))
    want[:, :u_ref.shape[1]] = u_ref[toks] * np.asarray(w["scales"], dtype=np.float64)[w["ids"][toks]][:, None]
    got = to_host(u[:T_lora])
    pad = np.arange(u.shape[1])[None, :] >= ranks[:, None]
    assert np.all(got[pad] == 0.0), tag + " u_save: padding ranks are not zero"
    assert_close(got, want, tag + " u_save")


def _check_layer(oracle, w, bwd, out_dtype=torch.float32, tol=(1e-2, 1e-3), tag="", table=False):
    y_ref, dX_ref, dA_ref, dB_ref = _oracle_all(oracle, w, bwd)
    L = HipLayer(w, out_dtype=out_dtype, want_bwd=bwd, table=str(table).startswith("table"), packed=str(table).endswith("packed"))
    y, u = L.fwd(save_u=bwd)
    stats = {"y": assert_close(to_host(y), y_ref, tag + " y", *tol)}
    if bwd:
        check_u_save(oracle, w, L, u, tag)
        for saved in (u, None):      # with the saved intermediate, then recomputing it
            dX, dA, dB = L.bwd(u_saved=saved)
            stats["dX"] = assert_close(to_host(dX), dX_ref, tag + " dX", *tol)
            for t in range(L.n):
                assert_close(to_host(dA[t]), dA_ref[t], tag + " dA[%d]" % t, *tol)
                assert_close(to_host(dB[t]), dB_ref[t], tag + " dB[%d]" % t, *tol)
    return stats


# ------------------------------------------------------------------ segment map
@pytest.mark.parametrize("T,n,neg", [(0, 4, False), (1, 1, False), (64, 4, False), (256, 32, True),
                                     (5000, 7, True), (16896, 64, False), (70000, 300, True)])
def test_segmap_matches_stable_argsort(T, n, neg):
    rng = np.random.default_rng(T + n)
    ids = rng.integers(-1 if neg else 0, n, size=T).astype(np.int32)
    if n > 2:
        ids[ids == 1] = 0        # adapter 1 stays empty
    ctx = api.marlaas_create(0)
    m = api.marlaas_segmap_build(ctx, torch.from_numpy(ids).cuda(), n)
    perm, seg_off = api.marlaas_segmap_export(m)
    key = np.where(ids < 0, n, ids)
    assert np.array_equal(perm, np.argsort(key, kind="stable").astype(np.int32))
    counts = np.bincount(key, minlength=n + 1)
    assert np.array_equal(seg_off, np.concatenate([[0], np.cumsum(counts)]).astype(np.int32))


def test_segmap_rejects_bad_ids():
    ctx = api.marlaas_create(0)
    for bad in (4, -2):
        ids = torch.tensor([0, 1, bad, 3], dtype=torch.int32, device="cuda")
        with pytest.raises(api.MarlaasError) as e:
            api.marlaas_segmap_build(ctx, ids, 4)
        assert e.value.status == -1


# ------------------------------------------------------------------ config 0 (fp32)
@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_config0_fp32(oracle, layout, seed):
    w = wl.make_config(0, seed=seed, layout=layout, want_dY=True)
    _check_layer(oracle, w, bwd=True, tol=(1e-4, 1e-5), tag="cfg0")


# ------------------------------------------------------------------ bf16 configs, reduced sizes
@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("cfg,scale", [(1, 0.25), (2, 0.05), (3, 0.03), (4, 0.08)])
def test_bf16_configs_scaled(oracle, cfg, scale, layout, use_table):
    w = wl.make_config(cfg, seed=cfg, scale=scale, layout=layout, want_dY=True)
    _check_layer(oracle, w, bwd=True, tag="cfg%d@%g" % (cfg, scale), table=use_table)


@pytest.mark.parametrize("layout", [0, 1])
def test_bf16_output_dtype(oracle, layout):
    """bf16 outputs: the final rounding alone costs up to 2^-9 relative, so the
    mean bound is the one of the metric with that floor added."""
    w = wl.make_config(4, seed=7, scale=0.05, layout=layout, want_dY=True)
    _check_layer(oracle, w, bwd=True, out_dtype=torch.bfloat16, tol=(1e-2, 2.5e-3), tag="bf16out")


# ------------------------------------------------------------------ config 1 at full size
@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_config1_full(oracle, layout, seed, use_table):
    w = wl.make_config(1, seed=seed, layout=layout)
    _check_layer(oracle, w, bwd=False, tag="cfg1", table=use_table)


@pytest.mark.parametrize("layout", [0, 1])
def test_config1_full_saves_u(oracle, layout, use_table):
    """The decode configuration with u_save requested: the fused shrink writes it from the finish kernel."""
    w = wl.make_config(1, seed=0, layout=layout)
    L = HipLayer(w, table=use_table.startswith("table"), packed=use_table.endswith("packed"))
    y, u = L.fwd(save_u=True)
    check_u_save(oracle, w, L, u, "cfg1")


# ------------------------------------------------------------------ ragged shapes and odd ranks
@pytest.mark.parametrize("layout", [0, 1])
def test_ragged_shapes_and_ranks(oracle, layout, use_table):
    rng = np.random.default_rng(5)
    ranks = [1, 5, 12, 100, 128, 16, 7]
    T = 777
    ids = rng.integers(-1, len(ranks), size=T).astype(np.int32)
    ids[ids == 5] = 2    # adapter 5 empty
    w = wl.make_layer(13, T, 520, 328, ranks, [2.0, 0.5, 1.0, 0.25, 0.125, 1.0, 3.0], ids,
                      dtype="bf16", layout=layout, want_dY=True)
    _check_layer(oracle, w, bwd=True, tag="ragged", table=use_table)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("ranks", [(8, 40, 64), (5, 12, 100), (128, 16)])
def test_long_segments_ragged_contraction(oracle, layout, ranks):
    """Around a thousand rows per adapter (the shrink then moves both operands by DMA through a ring
    of k-tiles, for factors stored rank-major with any rank, for factors stored contraction-major
    with ranks that are multiples of 8; odd ranks there take the register-staged kernel), 520 and
    328 features (a partial last k-tile in both passes), ragged segment lengths, rows without an
    adapter, ranks whose padded size is not a power of two."""
    rng = np.random.default_rng(19 + len(ranks))
    T = 1100 * len(ranks)
    ids = rng.integers(-1, len(ranks), size=T).astype(np.int32)
    w = wl.make_layer(53, T, 520, 328, list(ranks), [2.0, 0.5, 1.0][:len(ranks)], ids, dtype="bf16", layout=layout, want_dY=True)
    L = HipLayer(w, want_bwd=True)
    y, u = L.fwd(save_u=True)
    args = (w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"])
    assert_close(to_host(y), oracle.fwd(*args, layout=layout), "y")
    check_u_save(oracle, w, L, u, "long segments")
    dX, dA, dB = L.bwd(u_saved=u)
    dX_ref, dA_ref, dB_ref = oracle.bwd(*args, w["dY"], layout=layout)
    dA_ref, dB_ref = oracle_grads_in_layout(dA_ref, dB_ref, layout)
    assert_close(to_host(dX), dX_ref, "dX")
    for t in range(len(ranks)):
        assert_close(to_host(dA[t]), dA_ref[t], "dA[%d]" % t)
        assert_close(to_host(dB[t]), dB_ref[t], "dB[%d]" % t)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("ranks", [(8, 16, 24, 32), (1, 5, 12, 16, 7), (64, 64)])
def test_small_batch_paths(oracle, layout, ranks, use_table):
    """Few rows: the GEMM splits the contraction and, when the summed ranks fit its extended
    columns (and, for operands stored output-contiguous, every rank is a multiple of 8),
    computes the shrink itself; otherwise the separate shrink kernel runs.  The three rank sets
    take the fused path in both layouts, in one layout only, and in neither (128 > 96 columns).
    d_in = 520 leaves a contraction tail, T = 200 a ragged row tile, some rows have no adapter."""
    rng = np.random.default_rng(21)
    T = 200
    ids = rng.integers(-1, len(ranks), size=T).astype(np.int32)
    w = wl.make_layer(17, T, 520, 384, list(ranks), [1.0 + 0.5 * i for i in range(len(ranks))], ids,
                      dtype="bf16", layout=layout, want_dY=True)
    _check_layer(oracle, w, bwd=True, tag="small%s" % (ranks,), table=use_table)


def _padded(t, pad):
    """The same values as a view into a wider row-major buffer (leading dimension = width + pad)."""
    buf = torch.full((t.shape[0], t.shape[1] + pad), float("nan"), dtype=t.dtype, device=t.device)
    buf[:, :t.shape[1]] = t
    return buf[:, :t.shape[1]]


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("T", [96, 1500])
def test_padded_leading_dimensions(oracle, layout, T):
    """x, W, dY, y and dX as views into wider buffers (leading dimensions larger than the row
    length, padding filled with NaN): one row tile of the small-batch kernel (T = 96) and a dozen
    (T = 1500)."""
    rng = np.random.default_rng(9)
    ranks = [16, 8, 32]
    ids = rng.integers(-1, len(ranks), size=T).astype(np.int32)
    w = wl.make_layer(29, T, 328, 1032, ranks, [2.0, 1.0, 0.5], ids, dtype="bf16", layout=layout, want_dY=True)
    y_ref, dX_ref, dA_ref, dB_ref = _oracle_all(oracle, w, True)
    L = HipLayer(w, want_bwd=True)
    L.x, L.W, L.dY = _padded(L.x, 24), _padded(L.W, 8), _padded(L.dY, 40)
    L.desc = api.LoraDesc(L.x, L.W, L.A, L.B, w["ranks"], w["scales"], L.map, layout=layout, out_dtype=torch.float32)
    ybuf = torch.full((T, L.N + 16), float("nan"), dtype=torch.float32, device="cuda")
    dxbuf = torch.full((T, L.K + 8), float("nan"), dtype=torch.float32, device="cuda")
    y, dX = ybuf[:, :L.N], dxbuf[:, :L.K]
    dA = [torch.full(tuple(a.shape), float("nan"), dtype=torch.float32, device="cuda") for a in L.A]
    dB = [torch.full(tuple(b.shape), float("nan"), dtype=torch.float32, device="cuda") for b in L.B]
    api.marlaas_lora_fwd(L.ctx, L.desc, y)
    api.marlaas_lora_bwd(L.ctx, L.desc, L.dY, dX=dX, dA=dA, dB=dB)
    torch.cuda.synchronize()
    assert_close(to_host(y.contiguous()), y_ref, "ld y")
    assert_close(to_host(dX.contiguous()), dX_ref, "ld dX")
    assert bool(torch.isnan(ybuf[:, L.N:]).all()) and bool(torch.isnan(dxbuf[:, L.K:]).all())   # padding untouched
    for t in range(L.n):
        assert_close(to_host(dA[t]), dA_ref[t], "ld dA[%d]" % t)
        assert_close(to_host(dB[t]), dB_ref[t], "ld dB[%d]" % t)


@pytest.mark.parametrize("layout", [0, 1])
def test_many_adapters_few_tokens_each(oracle, layout, use_table):
    """300 adapters (ranks 4, 8, 12, 16 in turn) over 700 tokens: most segments hold one to four
    tokens, some adapters none; exercises the per-adapter grids and the row-chunk list."""
    rng = np.random.default_rng(41)
    n, T = 300, 700
    ranks = [4 * (1 + t % 4) for t in range(n)]
    ids = rng.integers(-1, n, size=T).astype(np.int32)
    w = wl.make_layer(37, T, 256, 384, ranks, [1.0 + (t % 3) for t in range(n)], ids, dtype="bf16", layout=layout, want_dY=True)
    _check_layer(oracle, w, bwd=True, tag="n300", table=use_table)


def test_hip_graph_replay_matches_eager():
    """Forward + backward captured once into a HIP graph (after an eager call)
    and replayed three times, with eager work and synchronisations between
    the replays: every replay reproduces the eager results bit for bit (this small batch takes
    the paths without atomics), also after the inputs changed in place."""
    rng = np.random.default_rng(3)
    ranks = [16, 8, 32, 16]
    T = 192
    ids = rng.integers(-1, len(ranks), size=T).astype(np.int32)
    w = wl.make_layer(5, T, 512, 640, ranks, [2.0, 1.0, 0.5, 2.0], ids, dtype="bf16", layout=wl.TORCH, want_dY=True)
    L = HipLayer(w, want_bwd=True)
    y = torch.empty((T, L.N), dtype=torch.float32, device="cuda")
    u = torch.zeros((T, api.marlaas_u_stride(L.desc)), dtype=torch.float32, device="cuda")
    dX = torch.empty((T, L.K), dtype=torch.float32, device="cuda")
    dA = [torch.empty(tuple(a.shape), dtype=torch.float32, device="cuda") for a in L.A]
    dB = [torch.empty(tuple(b.shape), dtype=torch.float32, device="cuda") for b in L.B]

    def step():
        api.marlaas_lora_fwd(L.ctx, L.desc, y, u_save=u)
        api.marlaas_lora_bwd(L.ctx, L.desc, L.dY, dX=dX, dA=dA, dB=dB, u_saved=u)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in [y, dX] + dA + dB]

    step()
    eager = snapshot()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    for rep in range(3):
        for t in [y, dX] + dA + dB:
            t.fill_(float("nan"))
        if rep == 2:                       # new input values in the same buffers
            L.x.mul_(0.5)
            step()
            eager = snapshot()
            for t in [y, dX] + dA + dB:
                t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        assert all(torch.equal(a, b) for a, b in zip(got, eager)), "replay %d differs from the eager pass" % rep
        (L.x.float() @ L.W.float().t()).sum().item()     # unrelated eager work between replays


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_random_shapes(oracle, seed, use_table):
    """Three seeded random problems per seed: T from a list that straddles the tile heights, d_in
    and d_out any multiples of 8 up to 1272, 0-9 adapters with ranks from 1 to 128, either
    layout, token order shuffled or grouped; forward and backward (with and without the saved
    intermediate) against the oracle."""
    rng = np.random.default_rng(100 + seed)
    for case in range(3):
        T = int(rng.choice([1, 2, 7, 16, 63, 64, 65, 128, 200, 257, 511, 900, 1300, 2049]))
        K, N = 8 * int(rng.integers(1, 160)), 8 * int(rng.integers(1, 160))
        n = int(rng.integers(0, 10))
        ranks = [int(rng.choice([1, 3, 4, 8, 16, 24, 32, 40, 64, 128])) for _ in range(n)]
        scales = [float(rng.choice([0.25, 0.5, 1.0, 2.0])) for _ in range(n)]
        layout = int(rng.integers(0, 2))
        ids = rng.integers(-1, max(n, 1), size=T).astype(np.int32) if n else np.full(T, -1, np.int32)
        if rng.random() < 0.3:
            ids = np.sort(ids)
        w = wl.make_layer(1000 * seed + case, T, K, N, ranks, scales, ids, dtype="bf16", layout=layout, want_dY=True)
        _check_layer(oracle, w, bwd=True, tag="rand s%d c%d T=%d K=%d N=%d ranks=%s layout=%d" % (seed, case, T, K, N, ranks, layout),
                     table=use_table)


def test_no_adapters_and_all_base_tokens(oracle):
    w = wl.make_layer(3, 300, 256, 512, [], [], np.full(300, -1, np.int32), dtype="bf16", want_dY=True)
    L = HipLayer(w, want_bwd=True)
    y, _ = L.fwd()
    y_ref = oracle.fwd(w["x"], w["W"], [], [], [], [], w["ids"])
    assert_close(to_host(y), y_ref, "n=0 y")
    dX, _, _ = L.bwd(want_grads=False)
    dX_ref, _, _ = oracle.bwd(w["x"], w["W"], [], [], [], [], w["ids"], w["dY"])
    assert_close(to_host(dX), dX_ref, "n=0 dX")
    # adapters exist but every token is base-only: gradients must be zero, y unchanged
    w2 = wl.make_layer(3, 300, 256, 512, [8, 16], [2.0, 2.0], np.full(300, -1, np.int32), dtype="bf16", want_dY=True)
    L2 = HipLayer(w2, want_bwd=True)
    y2, _ = L2.fwd()
    assert torch.equal(y2, y)
    _, dA, dB = L2.bwd()
    assert all(float(g.abs().max()) == 0.0 for g in dA + dB)


def test_zero_B_is_bitwise_base_only():
    """With B_t = 0 the fused extra steps add exact zeros: y must equal the
    base-only result bit for bit."""
    w = wl.make_config(4, seed=1, scale=0.05)
    w0 = dict(w, B=[np.zeros_like(b) for b in w["B"]])
    wb = dict(w, ids=np.full_like(w["ids"], -1))
    y0, _ = HipLayer(w0).fwd()
    yb, _ = HipLayer(wb).fwd()
    assert torch.equal(y0, yb)


def test_permutation_equivariance_on_gpu():
    """Permuting the tokens together with their labels permutes y and dX and leaves dA_t, dB_t
    unchanged (up to the summation order inside a segment)."""
    w = wl.make_config(4, seed=2, scale=0.04, want_dY=True)
    perm = np.random.default_rng(0).permutation(w["T"])
    wp = dict(w, x=np.ascontiguousarray(w["x"][perm]), dY=np.ascontiguousarray(w["dY"][perm]), ids=w["ids"][perm])
    L, Lp = HipLayer(w, want_bwd=True), HipLayer(wp, want_bwd=True)
    y, u = L.fwd(save_u=True)
    yp, up = Lp.fwd(save_u=True)
    assert_close(to_host(yp), to_host(y)[perm], "perm y", 1e-5, 1e-6)
    dX, dA, dB = L.bwd(u_saved=u)
    dXp, dAp, dBp = Lp.bwd(u_saved=up)
    assert_close(to_host(dXp), to_host(dX)[perm], "perm dX", 1e-5, 1e-6)
    for t in range(L.n):
        assert_close(to_host(dAp[t]), to_host(dA[t]), "perm dA[%d]" % t, 1e-4, 1e-5)
        assert_close(to_host(dBp[t]), to_host(dB[t]), "perm dB[%d]" % t, 1e-4, 1e-5)


def test_accumulate_and_empty_tokens(oracle):
    w = wl.make_config(4, seed=3, scale=0.04, want_dY=True)
    L = HipLayer(w, want_bwd=True)
    _, dA0, dB0 = L.bwd(want_dX=False)
    _, dA1, dB1 = L.bwd(want_dX=False, accumulate=True, init=1.0)
    for a0, a1 in zip(dA0 + dB0, dA1 + dB1):
        assert float((a1 - 1.0 - a0).abs().max()) <= 1e-5 * max(1.0, float(a0.abs().max()))
    # T = 0: forward is a no-op, backward zero-fills the gradients
    w0 = wl.make_layer(1, 0, 64, 64, [8], [1.0], np.zeros(0, np.int32), dtype="bf16", want_dY=True)
    L0 = HipLayer(w0, want_bwd=True)
    L0.fwd()
    _, dA, dB = L0.bwd()
    assert float(dA[0].abs().max()) == 0.0 and float(dB[0].abs().max()) == 0.0


def test_argument_errors_are_reported():
    w = wl.make_layer(1, 32, 64, 64, [8], [1.0], np.zeros(32, np.int32), dtype="bf16")
    L = HipLayer(w)
    y = torch.empty((32, 64), dtype=torch.float32, device="cuda")
    lib = api.load()
    ok = L.desc.c
    def status(**kw):
        import copy, ctypes
        c = api.marlaas_lora_desc.from_buffer_copy(ok)
        for k, v in kw.items():
            setattr(c, k, v)
        return lib.marlaas_lora_fwd(L.ctx.handle, ctypes.byref(c), y.data_ptr(), 64, None,
                                    torch.cuda.current_stream().cuda_stream)
    assert status() == 0
    assert status(x=None) == -1
    assert status(d_in=60) == -3
    assert status(x=ok.x + 2) == -3
    assert status(ldx=32) == -3
    assert status(T=31) == -2
    assert status(in_dtype=7) == -1
    bad_rank = (api.ctypes.c_int32 * 1)(0)
    assert status(ranks=api.ctypes.cast(bad_rank, api.ctypes.POINTER(api.ctypes.c_int32))) == -1
    api.marlaas_set_workspace(L.ctx, None)
    assert status() == -4
    assert b"workspace" in lib.marlaas_last_error(L.ctx.handle)
    torch.cuda.synchronize()


@pytest.mark.parametrize("layout", [0, 1])
def test_results_do_not_depend_on_timing(oracle, layout):
    """Few rows per adapter against a deep contraction, odd ranks: the shrink runs as its own kernel
    with its contraction split over workgroups, and the reductions split their tokens.  Every such
    sum is added up in a fixed order: three runs give the same bits in y, u, dX, dA, dB."""
    rng = np.random.default_rng(77)
    ranks = [5, 12, 7, 16, 3, 9]
    T = 700
    ids = rng.integers(-1, len(ranks), size=T).astype(np.int32)
    w = wl.make_layer(91, T, 4096, 264, ranks, [2.0, 0.5, 1.0, 0.25, 1.0, 3.0], ids, dtype="bf16", layout=layout, want_dY=True)
    L = HipLayer(w, want_bwd=True)
    runs = []
    for _ in range(3):
        y, u = L.fwd(save_u=True)
        dX, dA, dB = L.bwd(u_saved=u)
        runs.append([t.clone() for t in [y, u, dX] + list(dA) + list(dB)])
    for other in runs[1:]:
        for a, b in zip(runs[0], other):
            assert torch.equal(a, b)
    assert_close(to_host(runs[0][0]), oracle.fwd(w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"], layout=layout), "y")
