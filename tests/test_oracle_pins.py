"""Pins of the fp64 oracle against things other than itself: a hand-computed
example, exact rational brute force, library matmul on the merged dense weight,
structural invariants, finite differences and adjoint identities, and the
output variance the seeded init implies.  CPU only."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from harness import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))


def _f32_grid(rng, shape, std=1.0, bits=6):
    """float32 values on a coarse dyadic grid (so sums/differences with small
    dyadic steps stay exactly representable)."""
    q = 2.0 ** bits
    return (np.round(rng.standard_normal(shape) * std * q) / q).astype(np.float32)


def _tiny(rng, T=7, K=5, N=6, ranks=(3, 1, 2, 4), dtype="f32", layout=0, ids=None):
    n = len(ranks)
    if ids is None:
        ids = rng.integers(-1, n, size=T).astype(np.int32)
    mk = (lambda s, sd=1.0: _f32_grid(rng, s, sd)) if dtype == "f32" else \
         (lambda s, sd=1.0: wl.f32_to_bf16_bits(rng.standard_normal(s).astype(np.float32) * sd))
    x, W = mk((T, K)), mk((K, N), 0.5)
    A = [mk((K, r), 0.5) for r in ranks]
    B = [mk((r, N)) for r in ranks]
    dY = mk((T, N))
    scales = np.array([2.0, 0.5, 1.25, 3.0][:n], dtype=np.float32)
    if layout == 1:
        W = np.ascontiguousarray(W.T)
        A = [np.ascontiguousarray(a.T) for a in A]
        B = [np.ascontiguousarray(b.T) for b in B]
    return dict(x=x, W=W, A=A, B=B, ranks=np.array(ranks, np.int32), scales=scales, ids=ids, dY=dY,
                layout=layout)


def _call_fwd(oracle, p, **kw):
    return oracle.fwd(p["x"], p["W"], p["A"], p["B"], p["ranks"], p["scales"], p["ids"],
                      layout=p["layout"], **kw)


def _call_bwd(oracle, p, **kw):
    return oracle.bwd(p["x"], p["W"], p["A"], p["B"], p["ranks"], p["scales"], p["ids"], p["dY"],
                      layout=p["layout"], **kw)


def _math_view(p):
    """Widened (float64) tensors in math orientation."""
    tr = p["layout"] == 1
    W = wl.to_f64(p["W"]).T if tr else wl.to_f64(p["W"])
    A = [wl.to_f64(a).T if tr else wl.to_f64(a) for a in p["A"]]
    B = [wl.to_f64(b).T if tr else wl.to_f64(b) for b in p["B"]]
    return wl.to_f64(p["x"]), W, A, B, wl.to_f64(p["dY"])


# ---------------------------------------------------------------- hand example
def test_hand_example(oracle):
    g = json.load(open(os.path.join(HERE, "golden", "hand_example.json")))
    f = lambda a: np.array(a, dtype=np.float32)
    for layout in (0, 1):
        tr = (lambda a: np.ascontiguousarray(a.T)) if layout else (lambda a: a)
        args = (f(g["x"]), tr(f(g["W"])), [tr(f(a)) for a in g["A"]], [tr(f(b)) for b in g["B"]],
                g["ranks"], g["scales"], g["token_adapter"])
        y, u = oracle.fwd(*args, layout=layout, want_u=True)
        assert np.array_equal(y, np.array(g["y"]))
        assert np.array_equal(u, np.array(g["u"]))
        dX, dA, dB = oracle.bwd(*args, f(g["dY"]), layout=layout)
        assert np.array_equal(dX, np.array(g["dX"]))
        for t in range(2):
            assert np.array_equal(dA[t], np.array(g["dA"][t]))
            assert np.array_equal(dB[t], np.array(g["dB"][t]))


# ------------------------------------------------- exact rational brute force
def _brute(p):
    """Every output element as an exact rational, looping output-element-first
    (a different nest from the oracle's)."""
    x, W, A, B, dY = _math_view(p)
    F = lambda a: [[Fraction(float(v)) for v in row] for row in a]
    x, W, dY = F(x), F(W), F(dY)
    A, B = [F(a) for a in A], [F(b) for b in B]
    ids, ranks = p["ids"], p["ranks"]
    s = [Fraction(float(v)) for v in p["scales"]]
    T, K, N = len(x), len(W), len(W[0])
    y = [[None] * N for _ in range(T)]
    dX = [[None] * K for _ in range(T)]
    for i in range(T):
        t = ids[i]
        for j in range(N):
            acc = sum(x[i][k] * W[k][j] for k in range(K))
            if t >= 0:
                acc += s[t] * sum(sum(x[i][k] * A[t][k][q] for k in range(K)) * B[t][q][j]
                                  for q in range(ranks[t]))
            y[i][j] = acc
        for k in range(K):
            acc = sum(dY[i][j] * W[k][j] for j in range(N))
            if t >= 0:
                acc += sum(s[t] * sum(dY[i][j] * B[t][q][j] for j in range(N)) * A[t][k][q]
                           for q in range(ranks[t]))
            dX[i][k] = acc
    dA, dB = [], []
    for t in range(len(ranks)):
        seg = [i for i in range(T) if ids[i] == t]
        dA.append([[sum(x[i][k] * s[t] * sum(dY[i][j] * B[t][q][j] for j in range(N)) for i in seg)
                    for q in range(ranks[t])] for k in range(K)])
        dB.append([[s[t] * sum(sum(x[i][k] * A[t][k][q] for k in range(K)) * dY[i][j] for i in seg)
                    for j in range(N)] for q in range(ranks[t])])
    tof = lambda m: np.array([[float(v) for v in row] for row in m], dtype=np.float64).reshape(len(m), -1)
    return tof(y), tof(dX), [tof(a) for a in dA], [tof(b) for b in dB]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layout", [0, 1])
def test_brute_force_exact_rational(oracle, dtype, layout):
    rng = np.random.default_rng(11 + layout)
    # adapter 1 has rank 1, adapter 3 is empty, two tokens have no adapter
    ids = np.array([0, 2, -1, 1, 0, 2, -1, 1], dtype=np.int32)
    p = _tiny(rng, T=8, K=6, N=5, ranks=(3, 1, 2, 4), dtype=dtype, layout=layout, ids=ids)
    y, dX, dA, dB = _brute(p)
    oy = _call_fwd(oracle, p)
    odX, odA, odB = _call_bwd(oracle, p)
    tol = lambda ref: 1e-13 * max(1.0, np.abs(ref).max())
    assert np.abs(oy - y).max() <= tol(y)
    assert np.abs(odX - dX).max() <= tol(dX)
    for t in range(4):
        assert odA[t].shape == dA[t].shape and odB[t].shape == dB[t].shape
        assert np.abs(odA[t] - dA[t]).max() <= tol(dA[t])
        assert np.abs(odB[t] - dB[t]).max() <= tol(dB[t])
    assert np.all(odA[3] == 0) and np.all(odB[3] == 0)


# ------------------------------------------------------- structural invariants
def test_zero_B_is_exactly_base(oracle):
    rng = np.random.default_rng(3)
    p = _tiny(rng, T=33, K=40, N=24, dtype="bf16")
    p0 = dict(p, B=[np.zeros_like(b) for b in p["B"]])
    none = dict(p, ids=np.full(33, -1, np.int32))
    assert np.array_equal(_call_fwd(oracle, p0), _call_fwd(oracle, none))
    x, W, _, _, _ = _math_view(p)
    assert np.abs(_call_fwd(oracle, none) - x @ W).max() < 1e-12
    assert not np.array_equal(_call_fwd(oracle, p), _call_fwd(oracle, none))


@pytest.mark.parametrize("layout", [0, 1])
def test_single_adapter_equals_dense_merged_weight(oracle, layout):
    wlk = wl.make_layer(5, 48, 96, 80, [8], [2.0], np.zeros(48, np.int32), dtype="bf16",
                        layout=layout, want_dY=True)
    p = dict(wlk)
    x, W, A, B, dY = _math_view(p)
    s = 2.0
    merged = W + s * (A[0] @ B[0])
    y = _call_fwd(oracle, p)
    assert np.abs(y - x @ merged).max() <= 1e-12 * np.abs(y).max()
    dX, dA, dB = _call_bwd(oracle, p)
    assert np.abs(dX - dY @ merged.T).max() <= 1e-12 * np.abs(dX).max()
    # dense-layer weight gradient G = x^T dY projected on the factors
    G = x.T @ dY
    assert np.abs(dA[0] - s * G @ B[0].T).max() <= 1e-11 * np.abs(dA[0]).max()
    assert np.abs(dB[0] - s * A[0].T @ G).max() <= 1e-11 * np.abs(dB[0]).max()


@pytest.mark.parametrize("layout", [0, 1])
def test_matches_numpy_matmul_per_segment(oracle, layout):
    rng = np.random.default_rng(9)
    n, T = 5, 200
    ids = rng.integers(-1, n, size=T).astype(np.int32)
    ids[ids == 3] = 1  # adapter 3 has no tokens
    ranks = [4, 16, 1, 8, 5]
    scales = [2.0, 0.5, 1.0, 4.0, 0.25]
    p = wl.make_layer(21, T, 72, 56, ranks, scales, ids, dtype="bf16", layout=layout, want_dY=True)
    x, W, A, B, dY = _math_view(p)
    y, u = _call_fwd(oracle, p, want_u=True)
    dX, dA, dB = _call_bwd(oracle, p)
    for t in range(-1, n):
        m = ids == t
        if t < 0:
            assert np.abs(y[m] - x[m] @ W).max() < 1e-12
            assert np.abs(dX[m] - dY[m] @ W.T).max() < 1e-12
            continue
        ut = x[m] @ A[t]
        vt = scales[t] * dY[m] @ B[t].T
        assert np.abs(u[m][:, :ranks[t]] - ut).max() < 1e-12 if m.any() else True
        assert np.abs(y[m] - (x[m] @ W + scales[t] * ut @ B[t])).max() < 1e-11 if m.any() else True
        assert np.abs(dX[m] - (dY[m] @ W.T + vt @ A[t].T)).max() < 1e-11 if m.any() else True
        assert np.abs(dA[t] - x[m].T @ vt).max() < 1e-11
        assert np.abs(dB[t] - scales[t] * ut.T @ dY[m]).max() < 1e-11
    assert np.all(dA[3] == 0) and np.all(dB[3] == 0)


def test_layouts_agree(oracle):
    rng = np.random.default_rng(2)
    ids = rng.integers(-1, 3, size=20).astype(np.int32)
    a = wl.make_layer(4, 20, 24, 16, [2, 4, 8], [1.0, 2.0, 0.5], ids, dtype="bf16", layout=0, want_dY=True)
    b = wl.make_layer(4, 20, 24, 16, [2, 4, 8], [1.0, 2.0, 0.5], ids, dtype="bf16", layout=1, want_dY=True)
    assert np.array_equal(_call_fwd(oracle, a), _call_fwd(oracle, b))
    ra, rb = _call_bwd(oracle, a), _call_bwd(oracle, b)
    assert np.array_equal(ra[0], rb[0])
    for t in range(3):
        assert np.array_equal(ra[1][t], rb[1][t]) and np.array_equal(ra[2][t], rb[2][t])


def test_permutation_equivariance(oracle):
    rng = np.random.default_rng(8)
    p = _tiny(rng, T=40, K=24, N=16, dtype="bf16")
    perm = rng.permutation(40)
    q = dict(p, x=np.ascontiguousarray(p["x"][perm]), dY=np.ascontiguousarray(p["dY"][perm]),
             ids=p["ids"][perm])
    assert np.array_equal(_call_fwd(oracle, p)[perm], _call_fwd(oracle, q))
    dXp, dAp, dBp = _call_bwd(oracle, p)
    dXq, dAq, dBq = _call_bwd(oracle, q)
    assert np.array_equal(dXp[perm], dXq)
    for t in range(4):
        assert np.abs(dAp[t] - dAq[t]).max() <= 1e-13 * max(1.0, np.abs(dAp[t]).max())
        assert np.abs(dBp[t] - dBq[t]).max() <= 1e-13 * max(1.0, np.abs(dBp[t]).max())


def test_row_subset_matches_full(oracle):
    rng = np.random.default_rng(1)
    p = _tiny(rng, T=30, K=16, N=24, dtype="bf16")
    rows = np.array([29, 0, 7, 7, 13], dtype=np.int64)
    assert np.array_equal(_call_fwd(oracle, p)[rows], _call_fwd(oracle, p, rows=rows))
    full = _call_bwd(oracle, p)
    sub = _call_bwd(oracle, p, rows=rows, adapters=[2, 0])
    assert np.array_equal(full[0][rows], sub[0])
    assert np.array_equal(full[1][2], sub[1][0]) and np.array_equal(full[2][0], sub[2][1])


def test_linearity_and_scale(oracle):
    rng = np.random.default_rng(5)
    p = _tiny(rng, T=12, K=10, N=9, dtype="f32")
    x2 = _f32_grid(rng, p["x"].shape)
    y1 = _call_fwd(oracle, p)
    y2 = _call_fwd(oracle, dict(p, x=x2))
    y12 = _call_fwd(oracle, dict(p, x=(p["x"] + x2).astype(np.float32)))
    assert np.abs(y12 - (y1 + y2)).max() <= 1e-13 * np.abs(y12).max()
    base = _call_fwd(oracle, dict(p, ids=np.full(12, -1, np.int32)))
    yd = _call_fwd(oracle, dict(p, scales=(2 * p["scales"]).astype(np.float32)))
    assert np.abs((yd - base) - 2 * (y1 - base)).max() <= 1e-13 * np.abs(yd).max()


# ----------------------------------------------------------- gradient checks
def _loss(oracle, p):
    return float(np.sum(wl.to_f64(p["dY"]) * _call_fwd(oracle, p)))


@pytest.mark.parametrize("layout", [0, 1])
def test_gradients_match_central_differences(oracle, layout):
    """L = sum(dY * y) is linear in x, in each A_t and in each B_t, so a central
    difference with an exactly representable step is exact up to round-off."""
    rng = np.random.default_rng(17)
    p = _tiny(rng, T=9, K=7, N=6, ranks=(3, 1, 2, 4), dtype="f32", layout=layout)
    p["ids"] = np.array([0, 1, 2, -1, 0, 2, 2, 1, 0], np.int32)  # adapter 3 empty
    dX, dA, dB = _call_bwd(oracle, p)
    h = np.float32(2.0 ** -4)

    def fd(key, t, idx):
        vals = []
        for sgn in (+1, -1):
            q = dict(p)
            if t is None:
                arr = p[key].copy(); arr[idx] += sgn * h; q[key] = arr
            else:
                lst = [a.copy() for a in p[key]]; lst[t][idx] += sgn * h; q[key] = lst
            vals.append(_loss(oracle, q))
        return (vals[0] - vals[1]) / (2 * float(h))

    for i in range(9):
        for k in range(7):
            assert abs(fd("x", None, (i, k)) - dX[i, k]) <= 1e-9 * max(1.0, abs(dX[i, k]))
    for t, r in enumerate(p["ranks"]):
        for k in range(7):
            for q in range(r):
                idx = (q, k) if layout else (k, q)
                assert abs(fd("A", t, idx) - dA[t][k, q]) <= 1e-9 * max(1.0, abs(dA[t][k, q]))
        for q in range(r):
            for j in range(6):
                idx = (j, q) if layout else (q, j)
                assert abs(fd("B", t, idx) - dB[t][q, j]) <= 1e-9 * max(1.0, abs(dB[t][q, j]))


def test_adjoint_identities_config0_shape(oracle):
    """<dY, y(x+d)-y(x)> = <dX, d>, and the same for A and B, at the size of
    benchmark configuration 0 (values on a dyadic grid so x+d is exact)."""
    rng = np.random.default_rng(23)
    T, K, N, n, r = 64, 512, 512, 4, 8
    ids = rng.integers(0, n, size=T).astype(np.int32)
    p = dict(x=_f32_grid(rng, (T, K)), W=_f32_grid(rng, (K, N), K ** -0.5, 10),
             A=[_f32_grid(rng, (K, r), K ** -0.5, 10) for _ in range(n)],
             B=[_f32_grid(rng, (r, N), r ** -0.5, 8) for _ in range(n)],
             ranks=np.full(n, r, np.int32), scales=np.full(n, 2.0, np.float32), ids=ids,
             dY=_f32_grid(rng, (T, N)), layout=0)
    dX, dA, dB = _call_bwd(oracle, p)
    L0 = _loss(oracle, p)
    d = _f32_grid(rng, (T, K))
    lhs = _loss(oracle, dict(p, x=(p["x"] + d).astype(np.float32))) - L0
    assert abs(lhs - np.sum(dX * d)) <= 1e-10 * abs(lhs)
    dAs = [_f32_grid(rng, (K, r), 1.0, 10) for _ in range(n)]
    lhs = _loss(oracle, dict(p, A=[(a + e).astype(np.float32) for a, e in zip(p["A"], dAs)])) - L0
    assert abs(lhs - sum(np.sum(g * e) for g, e in zip(dA, dAs))) <= 1e-10 * abs(lhs)
    dBs = [_f32_grid(rng, (r, N), 1.0, 8) for _ in range(n)]
    lhs = _loss(oracle, dict(p, B=[(b + e).astype(np.float32) for b, e in zip(p["B"], dBs)])) - L0
    assert abs(lhs - sum(np.sum(g * e) for g, e in zip(dB, dBs))) <= 1e-10 * abs(lhs)


# ----------------------------------------------- statistics of the seeded init
def test_output_variance_of_seeded_init(oracle):
    """x~N(0,1), W~N(0,1/d_in), A~N(0,1/d_in), B~N(0,1/r) give Var[xW]=1,
    Var[u]=1, Var[uB]=1, hence Var[y] = 1 + s^2 for a token with an adapter."""
    ids = np.arange(600, dtype=np.int32) % 4
    ids[ids == 3] = -1
    p = wl.make_layer(0, 600, 256, 384, [8, 32, 16], [2.0, 0.5, 1.0], ids, dtype="bf16")
    y, u = _call_fwd(oracle, p, want_u=True)
    for t, s in ((-1, 0.0), (0, 2.0), (1, 0.5), (2, 1.0)):
        var = y[ids == t].var()
        assert abs(var / (1 + s * s) - 1) < 0.12, (t, var)
    assert abs(u[ids == 1][:, :32].var() - 1) < 0.1


def test_bad_token_id_is_an_error(oracle):
    rng = np.random.default_rng(0)
    p = _tiny(rng, dtype="f32")
    with pytest.raises(RuntimeError):
        _call_fwd(oracle, dict(p, ids=np.full(7, 4, np.int32)))
