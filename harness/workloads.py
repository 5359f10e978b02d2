"""Seeded synthetic inputs for the mixed-tenant multi-LoRA layer, and the error
metric used to compare an implementation with the fp64 oracle.

This module holds no arithmetic of the layer itself: it draws random tensors,
rounds them once to the storage type, and builds token->adapter maps.  Both the
oracle-side tests and the HIP-side tests/bench take their inputs from here, so
the two sides see bit-identical values.

Tensors are numpy arrays; bf16 tensors are uint16 bit patterns (round to
nearest even from fp32), fp32 tensors are float32.

The five workloads follow the benchmark configurations of this build:
  0  fp32 forward, T=64, 512x512, 4 adapters of rank 8, scale 2, ids uniform
  1  decode forward, bf16, T=256, 4096x4096, 32 adapters of rank 16, scale 2,
     ids ~ truncated Zipf(1.2) over the adapters, batch order unsorted
  2  prefill forward, bf16, d_in=4096, d_out=14336, 32 adapters of rank 16,
     1-8 sequences per adapter of length U[256,2048], rescaled to T=40960,
     contiguous segments
  3  training fwd+bwd, bf16, d_in=14336, d_out=4096, 16 adapters of rank 32,
     16384 tokens each, contiguous, dY ~ N(0,1)
  4  mixed fwd+bwd, bf16, 5120x5120, 64 adapters with ranks from {8,16,32,64},
     scale 16/r, 16384 prefill + 512 decode tokens, token-granular shuffle
Init for all: x~N(0,1), W~N(0,1/d_in), A_t~N(0,1/d_in), B_t~N(0,1/r_t).
"""
import os

import numpy as np

MATH, TORCH = 0, 1


def f32_to_bf16_bits(a):
    """Round float32 -> bf16 (nearest even), returned as uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    rnd = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(a):
    """Exact widening of a stored tensor (uint16 bf16 bits or float32)."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


_CHUNK = 1 << 22


def _normal(ss, shape, std, dtype):
    """N(0, std^2) drawn in fp32 and stored as `dtype`.  `ss` is a SeedSequence; every chunk of
    2^22 elements has its own child stream, so the values do not depend on the thread count."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16 if dtype == "bf16" else np.float32)
    nchunks = (n + _CHUNK - 1) // _CHUNK
    children = ss.spawn(nchunks) if nchunks else []

    def fill(i):
        s0, e0 = i * _CHUNK, min(n, (i + 1) * _CHUNK)
        c = np.random.Generator(np.random.PCG64(children[i])).standard_normal(e0 - s0, dtype=np.float32)
        if std != 1.0:
            c *= np.float32(std)
        out[s0:e0] = f32_to_bf16_bits(c) if dtype == "bf16" else c

    if nchunks <= 2:
        for i in range(nchunks):
            fill(i)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            list(ex.map(fill, range(nchunks)))
    return out.reshape(shape)


def zipf_ids(rng, T, n, s=1.2):
    """Each token's adapter ~ truncated Zipf: p(k) ~ (k+1)^-s, k = 0..n-1."""
    p = (np.arange(1, n + 1, dtype=np.float64)) ** (-s)
    p /= p.sum()
    return rng.choice(n, size=T, p=p).astype(np.int32)


def ragged_contiguous_ids(rng, n, T_total, seq_lo=256, seq_hi=2048, max_seqs=8):
    """1..max_seqs sequences per adapter with lengths U[seq_lo,seq_hi]; segment
    sizes rescaled so they add up to T_total exactly (every adapter keeps >= 1
    token); tokens of one adapter are contiguous, adapters in index order."""
    sizes = np.array([rng.integers(seq_lo, seq_hi + 1, size=rng.integers(1, max_seqs + 1)).sum()
                      for _ in range(n)], dtype=np.float64)
    if T_total is None:
        sz = sizes.astype(np.int64)
    else:
        sz = np.maximum(1, np.floor(sizes * (T_total / sizes.sum()))).astype(np.int64)
        d = int(T_total - sz.sum())
        order = np.argsort(-sizes, kind="stable")
        j = 0
        while d != 0:
            t = order[j % n]
            if d > 0:
                sz[t] += 1
                d -= 1
            elif sz[t] > 1:
                sz[t] -= 1
                d += 1
            j += 1
    return np.repeat(np.arange(n, dtype=np.int32), sz)


def make_layer(seed, T, d_in, d_out, ranks, scales, ids, dtype="bf16", layout=MATH, want_dY=False):
    """Draw x, W, A_t, B_t (and dY) for given shapes and token->adapter ids."""
    ranks = np.asarray(ranks, dtype=np.int32)
    n = len(ranks)
    stream = lambda *tag: np.random.SeedSequence([int(seed)] + [int(v) for v in tag])
    x = _normal(stream(0), (T, d_in), 1.0, dtype)
    W = _normal(stream(1), (d_in, d_out), d_in ** -0.5, dtype)
    A = [_normal(stream(2, t), (d_in, int(r)), d_in ** -0.5, dtype) for t, r in enumerate(ranks)]
    B = [_normal(stream(3, t), (int(r), d_out), float(r) ** -0.5, dtype) for t, r in enumerate(ranks)]
    dY = _normal(stream(4), (T, d_out), 1.0, dtype) if want_dY else None
    if layout == TORCH:
        W = np.ascontiguousarray(W.T)
        A = [np.ascontiguousarray(a.T) for a in A]
        B = [np.ascontiguousarray(b.T) for b in B]
    return dict(T=T, d_in=d_in, d_out=d_out, n_adapters=n, dtype=dtype, layout=layout,
                x=x, W=W, A=A, B=B, ranks=ranks,
                scales=np.asarray(scales, dtype=np.float32), ids=np.asarray(ids, dtype=np.int32),
                dY=dY)


def config_shape(cfg, scale=1.0):
    """Shape parameters of benchmark configuration `cfg`; scale < 1 shrinks the
    token count and the feature dims (kept multiples of 64) for quick tests."""
    def dim(d):
        return max(64, int(round(d * scale / 64)) * 64) if scale != 1.0 else d
    def tok(t):
        return max(8, int(round(t * scale))) if scale != 1.0 else t
    if cfg == 0:
        return dict(T=tok(64), d_in=dim(512), d_out=dim(512), n=4, dtype="f32", bwd=False)
    if cfg == 1:
        return dict(T=tok(256), d_in=dim(4096), d_out=dim(4096), n=32, dtype="bf16", bwd=False)
    if cfg == 2:
        return dict(T=tok(40960), d_in=dim(4096), d_out=dim(14336), n=32, dtype="bf16", bwd=False)
    if cfg == 3:
        return dict(T=16 * tok(16384), d_in=dim(14336), d_out=dim(4096), n=16, dtype="bf16", bwd=True)
    if cfg == 4:
        return dict(T=tok(16384) + tok(512), d_in=dim(5120), d_out=dim(5120), n=64, dtype="bf16", bwd=True)
    raise ValueError("config must be 0..4")


def config_ids(cfg, seed, scale=1.0):
    """ranks, scales and the token->adapter map of configuration `cfg`."""
    sh = config_shape(cfg, scale)
    rng = np.random.Generator(np.random.PCG64([seed, 1000 + cfg]))
    n, T = sh["n"], sh["T"]
    if cfg == 0:
        ranks = np.full(n, 8, np.int32)
        scales = np.full(n, 2.0, np.float32)
        ids = rng.integers(0, n, size=T).astype(np.int32)
    elif cfg == 1:
        ranks = np.full(n, 16, np.int32)
        scales = np.full(n, 2.0, np.float32)
        ids = zipf_ids(rng, T, n, 1.2)
    elif cfg == 2:
        ranks = np.full(n, 16, np.int32)
        scales = np.full(n, 2.0, np.float32)
        ids = ragged_contiguous_ids(rng, n, T)
    elif cfg == 3:
        ranks = np.full(n, 32, np.int32)
        scales = np.full(n, 2.0, np.float32)
        ids = np.repeat(np.arange(n, dtype=np.int32), T // n)
    else:
        ranks = rng.choice(np.array([8, 16, 32, 64], np.int32), size=n).astype(np.int32)
        scales = (16.0 / ranks).astype(np.float32)
        n_dec = max(1, int(round(512 * scale))) if scale != 1.0 else 512
        n_pre = T - n_dec
        lo, hi = (256, 2048) if scale == 1.0 else (max(1, int(256 * scale)), max(2, int(2048 * scale)))
        ids_list, tot = [], 0
        while tot < n_pre:
            L = min(int(rng.integers(lo, hi + 1)), n_pre - tot)
            ids_list.append(np.full(L, rng.integers(0, n), np.int32))
            tot += L
        ids_list.append(rng.integers(0, n, size=n_dec).astype(np.int32))
        ids = np.concatenate(ids_list)
        ids = ids[rng.permutation(T)]
    return sh, ranks, scales, ids


def make_config(cfg, seed=0, scale=1.0, layout=MATH, want_dY=None):
    sh, ranks, scales, ids = config_ids(cfg, seed, scale)
    want = sh["bwd"] if want_dY is None else want_dY
    wl = make_layer(seed, sh["T"], sh["d_in"], sh["d_out"], ranks, scales, ids,
                    dtype=sh["dtype"], layout=layout, want_dY=want)
    wl["config"] = cfg
    return wl


def rel_err_stats(got, ref):
    """Floored relative error of `got` against the oracle `ref` (both arrays of
    one output tensor): rel_i = |g_i - o_i| / max(|o_i|, rms(o)).  Returns
    (max rel, mean rel, ||g-o||_2 / ||o||_2).  An all-zero reference compares
    absolutely (rms floor replaced by 1)."""
    g = np.asarray(got, dtype=np.float64).ravel()
    o = np.asarray(ref, dtype=np.float64).ravel()
    assert g.shape == o.shape
    if o.size == 0:
        return 0.0, 0.0, 0.0
    rms = float(np.sqrt(np.mean(o * o)))
    floor = rms if rms > 0.0 else 1.0
    rel = np.abs(g - o) / np.maximum(np.abs(o), floor)
    nrm = float(np.linalg.norm(o))
    return float(rel.max()), float(rel.mean()), float(np.linalg.norm(g - o) / (nrm if nrm > 0 else 1.0))
