"""ctypes front-end of the fp64 CPU oracle in lora_oracle.c.

Test infrastructure only: imported by tests/, the smoke check and the
cpu_baseline leg of bench.py.  It imports nothing from the HIP package and the
HIP package imports nothing from here.

Arrays: bf16 tensors are numpy uint16 bit patterns, fp32 tensors numpy float32.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lora_oracle.c")
_SO = os.path.join(_HERE, "liblora_oracle.so")
_lib = None


def build(force=False):
    """Compile lora_oracle.c with gcc (fp64, OpenMP, no BLAS)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_SO)
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_fwd.restype = ctypes.c_int
        lib.oracle_bwd.restype = ctypes.c_int
        lib.oracle_adamw_step.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads():
    return int(_load().oracle_num_threads())


def _dtype_flag(arr):
    if arr.dtype == np.uint16:
        return 0
    if arr.dtype == np.float32:
        return 1
    raise TypeError("oracle inputs must be uint16 (bf16 bits) or float32, got %s" % arr.dtype)


def _ptr(arr):
    return ctypes.c_void_p(arr.ctypes.data)


def _ptr_array(arrs):
    return (ctypes.c_void_p * max(len(arrs), 1))(*[a.ctypes.data for a in arrs])


def _common(x, W, A, B, ranks, scales, token_adapter, layout):
    dt = _dtype_flag(x)
    for a in [W] + list(A) + list(B):
        if _dtype_flag(a) != dt:
            raise TypeError("mixed input dtypes")
    T, K = x.shape
    N = W.shape[1] if layout == 0 else W.shape[0]
    assert (W.shape == (K, N)) if layout == 0 else (W.shape == (N, K))
    n = len(A)
    ranks = np.ascontiguousarray(ranks, dtype=np.int32)
    scales = np.ascontiguousarray(scales, dtype=np.float64)
    ids = np.ascontiguousarray(token_adapter, dtype=np.int32)
    assert ids.shape == (T,) and len(B) == n and ranks.shape == (n,) and scales.shape == (n,)
    for t in range(n):
        r = int(ranks[t])
        assert A[t].flags.c_contiguous and B[t].flags.c_contiguous
        assert A[t].shape == ((K, r) if layout == 0 else (r, K)), (A[t].shape, K, r)
        assert B[t].shape == ((r, N) if layout == 0 else (N, r)), (B[t].shape, r, N)
    assert x.flags.c_contiguous and W.flags.c_contiguous
    return dt, T, K, N, n, ranks, scales, ids


def fwd(x, W, A, B, ranks, scales, token_adapter, layout=0, rows=None, want_u=False):
    """y (float64 [n_rows or T, d_out]) and optionally u (float64 [*, r_max])."""
    dt, T, K, N, n, ranks, scales, ids = _common(x, W, A, B, ranks, scales, token_adapter, layout)
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        assert rows.ndim == 1 and (rows.size == 0 or (rows.min() >= 0 and rows.max() < T))
    n_out = T if rows is None else rows.size
    r_max = int(ranks.max()) if n > 0 else 0
    y = np.zeros((n_out, N), dtype=np.float64)
    u = np.zeros((n_out, max(r_max, 1)), dtype=np.float64) if want_u else None
    rc = _load().oracle_fwd(
        ctypes.c_int(dt), ctypes.c_int(layout), ctypes.c_int64(T), ctypes.c_int64(K),
        ctypes.c_int64(N), ctypes.c_int(n), _ptr(x), ctypes.c_int64(x.strides[0] // x.itemsize),
        _ptr(W), ctypes.c_int64(W.strides[0] // W.itemsize), _ptr_array(A), _ptr_array(B),
        _ptr(ranks), _ptr(scales), _ptr(ids),
        _ptr(rows) if rows is not None else None, ctypes.c_int64(n_out), _ptr(y),
        _ptr(u) if want_u else None, ctypes.c_int64(r_max))
    if rc != 0:
        raise RuntimeError("oracle_fwd failed (bad token id or out of memory)")
    if want_u:
        return y, u[:, :r_max]
    return y


def bwd(x, W, A, B, ranks, scales, token_adapter, dY, layout=0, rows=None, want_dX=True,
        adapters=None):
    """dX (float64 [n_rows or T, d_in]) and, for every adapter index in
    `adapters` (default: all), dA_t as [d_in, r_t] and dB_t as [r_t, d_out]
    (math orientation whatever the input layout).  Returns (dX, dA, dB) with dA
    and dB lists aligned with `adapters`."""
    dt, T, K, N, n, ranks, scales, ids = _common(x, W, A, B, ranks, scales, token_adapter, layout)
    assert _dtype_flag(dY) == dt and dY.shape == (T, N) and dY.flags.c_contiguous
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        assert rows.ndim == 1 and (rows.size == 0 or (rows.min() >= 0 and rows.max() < T))
    n_out = T if rows is None else rows.size
    dX = np.zeros((n_out, K), dtype=np.float64) if want_dX else None
    sel = np.arange(n, dtype=np.int32) if adapters is None else np.ascontiguousarray(adapters, dtype=np.int32)
    assert sel.size == 0 or (sel.min() >= 0 and sel.max() < n)
    dA = [np.zeros((K, int(ranks[t])), dtype=np.float64) for t in sel]
    dB = [np.zeros((int(ranks[t]), N), dtype=np.float64) for t in sel]
    rc = _load().oracle_bwd(
        ctypes.c_int(dt), ctypes.c_int(layout), ctypes.c_int64(T), ctypes.c_int64(K),
        ctypes.c_int64(N), ctypes.c_int(n), _ptr(x), ctypes.c_int64(x.strides[0] // x.itemsize),
        _ptr(W), ctypes.c_int64(W.strides[0] // W.itemsize), _ptr_array(A), _ptr_array(B),
        _ptr(ranks), _ptr(scales), _ptr(ids), _ptr(dY), ctypes.c_int64(dY.strides[0] // dY.itemsize),
        _ptr(rows) if rows is not None else None, ctypes.c_int64(n_out),
        _ptr(dX) if want_dX else None,
        _ptr(sel), ctypes.c_int(sel.size), _ptr_array(dA), _ptr_array(dB))
    if rc != 0:
        raise RuntimeError("oracle_bwd failed (bad token id or out of memory)")
    return dX, dA, dB


def adamw_step(p, m, v, g, lr, beta1, beta2, eps, weight_decay, step):
    """One AdamW step in fp64 on arrays of any (equal) shape; `step` is the number of this update
    (1 for the first).  Returns new (p, m, v) as float64 arrays; the inputs are not modified."""
    p2, m2, v2 = (np.array(a, dtype=np.float64, order="C", copy=True) for a in (p, m, v))
    g2 = np.ascontiguousarray(g, dtype=np.float64)
    assert p2.shape == m2.shape == v2.shape == g2.shape
    rc = _load().oracle_adamw_step(
        ctypes.c_int64(p2.size), _ptr(p2), _ptr(m2), _ptr(v2), _ptr(g2), ctypes.c_double(lr),
        ctypes.c_double(beta1), ctypes.c_double(beta2), ctypes.c_double(eps), ctypes.c_double(weight_decay),
        ctypes.c_int64(step))
    if rc != 0:
        raise RuntimeError("oracle_adamw_step failed (step must be >= 1)")
    return p2, m2, v2
