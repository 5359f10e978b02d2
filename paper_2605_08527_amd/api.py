"""Python binding of libmarlaas_lora.so: argument marshalling only.

Every function here has the name of the C entry point it calls (see
include/marlaas_lora.h).  Tensors are torch CUDA tensors used purely as device
memory; all arithmetic happens inside the HIP library.  There is no fallback:
if the library is missing, loading raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("MARLAAS_LORA_LIB", os.path.join(_HERE, "libmarlaas_lora.so"))

MARLAAS_BF16, MARLAAS_F32 = 0, 1
MARLAAS_LAYOUT_MATH, MARLAAS_LAYOUT_TORCH = 0, 1
MARLAAS_OK = 0

EXPORTS = [
    "marlaas_create", "marlaas_destroy", "marlaas_strerror", "marlaas_last_error",
    "marlaas_segmap_build", "marlaas_segmap_destroy", "marlaas_segmap_export",
    "marlaas_segmap_create", "marlaas_segmap_update",
    "marlaas_adapter_table_create", "marlaas_adapter_table_destroy", "marlaas_adapter_table_update",
    "marlaas_adapter_table_version", "marlaas_adapter_table_plan_version",
    "marlaas_workspace_bytes", "marlaas_set_workspace", "marlaas_lora_fwd", "marlaas_lora_bwd", "marlaas_lora_bwd_adamw",
    "marlaas_lora_fwd_static", "marlaas_packed_weight_bytes", "marlaas_pack_weight", "marlaas_transpose_weight",
    "marlaas_workspace_bytes_multi", "marlaas_lora_fwd_multi",
    "marlaas_u_stride", "marlaas_profile_enable", "marlaas_profile_read",
]
MARLAAS_KERNEL_SHRINK, MARLAAS_KERNEL_GEMM, MARLAAS_KERNEL_REDUCE = 1, 2, 3


class marlaas_adamw(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
                ("weight_decay", ctypes.c_float), ("step", ctypes.c_int32)]


class marlaas_adapter_state(ctypes.Structure):
    _fields_ = [("master_A", ctypes.c_void_p), ("master_B", ctypes.c_void_p), ("m_A", ctypes.c_void_p),
                ("v_A", ctypes.c_void_p), ("m_B", ctypes.c_void_p), ("v_B", ctypes.c_void_p),
                ("A_next", ctypes.c_void_p), ("B_next", ctypes.c_void_p)]


class marlaas_lora_desc(ctypes.Structure):
    _fields_ = [
        ("T", ctypes.c_int64), ("d_in", ctypes.c_int64), ("d_out", ctypes.c_int64),
        ("n_adapters", ctypes.c_int32), ("in_dtype", ctypes.c_int32),
        ("out_dtype", ctypes.c_int32), ("layout", ctypes.c_int32),
        ("x", ctypes.c_void_p), ("ldx", ctypes.c_int64),
        ("W", ctypes.c_void_p), ("ldw", ctypes.c_int64),
        ("A", ctypes.POINTER(ctypes.c_void_p)), ("B", ctypes.POINTER(ctypes.c_void_p)),
        ("ranks", ctypes.POINTER(ctypes.c_int32)), ("scales", ctypes.POINTER(ctypes.c_float)),
        ("map", ctypes.c_void_p),
        ("table", ctypes.c_void_p), ("proj", ctypes.c_int32), ("reserved", ctypes.c_int32),
        ("W_packed_fwd", ctypes.c_void_p), ("W_packed_bwd", ctypes.c_void_p), ("W_t", ctypes.c_void_p),
    ]


_lib = None


def load():
    """dlopen the HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("%s is missing: run paper_2605_08527_amd/build.py (there is no fallback path)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.marlaas_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int]
    lib.marlaas_create.restype = ctypes.c_int
    lib.marlaas_destroy.argtypes = [vp]
    lib.marlaas_destroy.restype = None
    lib.marlaas_strerror.argtypes = [ctypes.c_int]
    lib.marlaas_strerror.restype = ctypes.c_char_p
    lib.marlaas_last_error.argtypes = [vp]
    lib.marlaas_last_error.restype = ctypes.c_char_p
    lib.marlaas_segmap_build.argtypes = [vp, vp, i64, i32, vp, ctypes.POINTER(vp)]
    lib.marlaas_segmap_build.restype = ctypes.c_int
    lib.marlaas_segmap_destroy.argtypes = [vp]
    lib.marlaas_segmap_destroy.restype = None
    lib.marlaas_segmap_export.argtypes = [vp, vp, vp]
    lib.marlaas_segmap_export.restype = ctypes.c_int
    lib.marlaas_segmap_create.argtypes = [vp, i64, i32, ctypes.POINTER(vp)]
    lib.marlaas_segmap_create.restype = ctypes.c_int
    lib.marlaas_segmap_update.argtypes = [vp, vp, vp, i64, i32, vp]
    lib.marlaas_segmap_update.restype = ctypes.c_int
    lib.marlaas_adapter_table_create.argtypes = [vp, i32, i32, i32, ctypes.POINTER(vp)]
    lib.marlaas_adapter_table_create.restype = ctypes.c_int
    lib.marlaas_adapter_table_destroy.argtypes = [vp]
    lib.marlaas_adapter_table_destroy.restype = None
    lib.marlaas_adapter_table_update.argtypes = [vp, vp, i32, i32, vp, vp, i32, ctypes.c_float, vp, vp, vp]
    lib.marlaas_adapter_table_update.restype = ctypes.c_int
    lib.marlaas_adapter_table_version.argtypes = [vp, i32, i32]
    lib.marlaas_adapter_table_version.restype = i64
    lib.marlaas_adapter_table_plan_version.argtypes = [vp]
    lib.marlaas_adapter_table_plan_version.restype = i64
    lib.marlaas_workspace_bytes.argtypes = [ctypes.POINTER(marlaas_lora_desc), ctypes.c_int]
    lib.marlaas_workspace_bytes.restype = ctypes.c_size_t
    lib.marlaas_set_workspace.argtypes = [vp, vp, ctypes.c_size_t]
    lib.marlaas_set_workspace.restype = ctypes.c_int
    lib.marlaas_lora_fwd.argtypes = [vp, ctypes.POINTER(marlaas_lora_desc), vp, i64, vp, vp]
    lib.marlaas_lora_fwd.restype = ctypes.c_int
    lib.marlaas_packed_weight_bytes.argtypes = [i64, i64, i32]
    lib.marlaas_packed_weight_bytes.restype = ctypes.c_size_t
    lib.marlaas_pack_weight.argtypes = [vp, vp, i64, i64, i64, i32, i32, vp, vp]
    lib.marlaas_pack_weight.restype = ctypes.c_int
    lib.marlaas_transpose_weight.argtypes = [vp, vp, i64, i64, i64, i32, vp, vp]
    lib.marlaas_transpose_weight.restype = ctypes.c_int
    lib.marlaas_lora_fwd_static.argtypes = [vp, ctypes.POINTER(marlaas_lora_desc), vp, i64, vp, vp]
    lib.marlaas_lora_fwd_static.restype = ctypes.c_int
    lib.marlaas_lora_bwd.argtypes = [vp, ctypes.POINTER(marlaas_lora_desc), vp, i64, vp, vp, i64,
                                     vp, vp, ctypes.c_int, vp]
    lib.marlaas_lora_bwd.restype = ctypes.c_int
    lib.marlaas_lora_bwd_adamw.argtypes = [vp, ctypes.POINTER(marlaas_lora_desc), vp, i64, vp, vp, i64,
                                           ctypes.POINTER(marlaas_adapter_state), ctypes.POINTER(marlaas_adamw), vp]
    lib.marlaas_lora_bwd_adamw.restype = ctypes.c_int
    lib.marlaas_workspace_bytes_multi.argtypes = [ctypes.POINTER(marlaas_lora_desc), i32]
    lib.marlaas_workspace_bytes_multi.restype = ctypes.c_size_t
    lib.marlaas_lora_fwd_multi.argtypes = [vp, ctypes.POINTER(marlaas_lora_desc), i32, ctypes.POINTER(ctypes.c_void_p),
                                           ctypes.POINTER(i64), vp]
    lib.marlaas_lora_fwd_multi.restype = ctypes.c_int
    lib.marlaas_u_stride.argtypes = [ctypes.POINTER(marlaas_lora_desc)]
    lib.marlaas_u_stride.restype = i64
    lib.marlaas_profile_enable.argtypes = [vp, ctypes.c_int]
    lib.marlaas_profile_enable.restype = ctypes.c_int
    lib.marlaas_profile_read.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    lib.marlaas_profile_read.restype = ctypes.c_int
    _lib = lib
    return lib


class MarlaasError(RuntimeError):
    def __init__(self, status, detail):
        self.status = status
        text = load().marlaas_strerror(status).decode()
        super().__init__("marlaas status %d (%s): %s" % (status, text, detail))


def _check(ctx, status):
    if status != MARLAAS_OK:
        detail = load().marlaas_last_error(ctx.handle).decode() if ctx is not None else ""
        raise MarlaasError(status, detail)


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _dtype_flag(dt):
    if dt == torch.bfloat16:
        return MARLAAS_BF16
    if dt == torch.float32:
        return MARLAAS_F32
    raise TypeError("only bfloat16 and float32 tensors are supported, got %s" % dt)


class Context:
    def __init__(self, device=0):
        self.handle = ctypes.c_void_p()
        self.workspace = None
        st = load().marlaas_create(ctypes.byref(self.handle), int(device))
        if st != MARLAAS_OK:
            raise MarlaasError(st, "marlaas_create(device=%d)" % device)

    def close(self):
        if self.handle:
            load().marlaas_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def marlaas_create(device=0):
    return Context(device)


def marlaas_destroy(ctx):
    ctx.close()


class Segmap:
    def __init__(self, handle, T, n_adapters):
        self.handle, self.T, self.n_adapters = handle, T, n_adapters

    def close(self):
        if self.handle:
            load().marlaas_segmap_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def marlaas_segmap_build(ctx, token_adapter, n_adapters, stream=None):
    """token_adapter: int32 CUDA tensor [T]."""
    assert token_adapter.dtype == torch.int32 and token_adapter.is_cuda and token_adapter.is_contiguous()
    h = ctypes.c_void_p()
    st = load().marlaas_segmap_build(ctx.handle, _ptr(token_adapter), token_adapter.numel(),
                                     int(n_adapters), _stream_ptr(stream), ctypes.byref(h))
    _check(ctx, st)
    return Segmap(h, token_adapter.numel(), int(n_adapters))


def marlaas_segmap_destroy(segmap):
    segmap.close()


def marlaas_segmap_create(ctx, T_max, n_adapters_max):
    """A map object with room for T_max tokens / n_adapters_max adapters (holds no map yet)."""
    h = ctypes.c_void_p()
    _check(ctx, load().marlaas_segmap_create(ctx.handle, int(T_max), int(n_adapters_max), ctypes.byref(h)))
    return Segmap(h, 0, 0)


def marlaas_segmap_update(ctx, segmap, token_adapter, n_adapters, stream=None):
    """Regroup a new batch into an existing map object (no allocation)."""
    assert token_adapter.dtype == torch.int32 and token_adapter.is_cuda and token_adapter.is_contiguous()
    _check(ctx, load().marlaas_segmap_update(ctx.handle, segmap.handle, _ptr(token_adapter), token_adapter.numel(),
                                             int(n_adapters), _stream_ptr(stream)))
    segmap.T, segmap.n_adapters = token_adapter.numel(), int(n_adapters)


MARLAAS_GRADS_IN_TABLE = ctypes.c_void_p(1)


class AdapterTable:
    """Owns a marlaas_adapter_table and keeps the registered tensors alive."""

    def __init__(self, handle, n_adapters, n_proj):
        self.handle, self.n_adapters, self.n_proj = handle, n_adapters, n_proj
        self.tensors = {}

    def close(self):
        if self.handle:
            load().marlaas_adapter_table_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def marlaas_adapter_table_create(ctx, n_adapters, n_proj=1, max_rank=128):
    h = ctypes.c_void_p()
    _check(ctx, load().marlaas_adapter_table_create(ctx.handle, int(n_adapters), int(n_proj), int(max_rank), ctypes.byref(h)))
    return AdapterTable(h, int(n_adapters), int(n_proj))


def marlaas_adapter_table_destroy(table):
    table.close()


def marlaas_adapter_table_update(ctx, table, proj, t, A, B, rank, scale, dA=None, dB=None, stream=None):
    _check(ctx, load().marlaas_adapter_table_update(ctx.handle, table.handle, int(proj), int(t), _ptr(A), _ptr(B), int(rank),
                                                    float(scale), _ptr(dA), _ptr(dB), _stream_ptr(stream)))
    table.tensors[(int(proj), int(t))] = (A, B, dA, dB)


def marlaas_adapter_table_version(table, proj=0, t=-1):
    return int(load().marlaas_adapter_table_version(table.handle, int(proj), int(t)))


def marlaas_adapter_table_plan_version(table):
    return int(load().marlaas_adapter_table_plan_version(table.handle))


def marlaas_segmap_export(segmap):
    """(perm, seg_off) as numpy int32 arrays."""
    import numpy as np
    perm = np.empty(segmap.T, dtype=np.int32)
    seg_off = np.empty(segmap.n_adapters + 2, dtype=np.int32)
    st = load().marlaas_segmap_export(segmap.handle, ctypes.c_void_p(perm.ctypes.data),
                                      ctypes.c_void_p(seg_off.ctypes.data))
    if st != MARLAAS_OK:
        raise MarlaasError(st, "marlaas_segmap_export")
    return perm, seg_off


class LoraDesc:
    """Owns a marlaas_lora_desc and keeps the host arrays it points to alive."""

    def __init__(self, x, W, A, B, ranks, scales, segmap, layout=MARLAAS_LAYOUT_MATH, out_dtype=None,
                 table=None, proj=0, W_packed_fwd=None, W_packed_bwd=None, W_t=None):
        """With `table` (an AdapterTable) the adapters come from the table's projection `proj` and
        A, B, ranks, scales are ignored (pass None).  W_packed_*: tensors written by marlaas_pack_weight."""
        if table is not None:
            A, B, ranks, scales = [], [], [], []
        n = len(A) if table is None else table.n_adapters
        self.tensors = (x, W, list(A), list(B), segmap, table)
        self.c = marlaas_lora_desc()
        T, d_in = x.shape
        d_out = W.shape[1] if layout == MARLAAS_LAYOUT_MATH else W.shape[0]
        self.c.T, self.c.d_in, self.c.d_out, self.c.n_adapters = T, d_in, d_out, n
        self.c.in_dtype = _dtype_flag(x.dtype)
        self.c.out_dtype = self.c.in_dtype if out_dtype is None else _dtype_flag(out_dtype)
        self.c.layout = layout
        self.c.x, self.c.ldx = x.data_ptr(), x.stride(0) if T > 0 else d_in
        self.c.W, self.c.ldw = W.data_ptr(), W.stride(0)
        self.c.table = table.handle if table is not None else None
        self.c.proj, self.c.reserved = int(proj), 0
        self.packed = (W_packed_fwd, W_packed_bwd, W_t)
        self.c.W_t = W_t.data_ptr() if W_t is not None else None
        self.c.W_packed_fwd = W_packed_fwd.data_ptr() if W_packed_fwd is not None else None
        self.c.W_packed_bwd = W_packed_bwd.data_ptr() if W_packed_bwd is not None else None
        self._A = (ctypes.c_void_p * max(n, 1))(*[a.data_ptr() for a in A])
        self._B = (ctypes.c_void_p * max(n, 1))(*[b.data_ptr() for b in B])
        self._ranks = (ctypes.c_int32 * max(n, 1))(*[int(r) for r in ranks])
        self._scales = (ctypes.c_float * max(n, 1))(*[float(s) for s in scales])
        self.c.A = ctypes.cast(self._A, ctypes.POINTER(ctypes.c_void_p))
        self.c.B = ctypes.cast(self._B, ctypes.POINTER(ctypes.c_void_p))
        self.c.ranks = ctypes.cast(self._ranks, ctypes.POINTER(ctypes.c_int32))
        self.c.scales = ctypes.cast(self._scales, ctypes.POINTER(ctypes.c_float))
        self.c.map = segmap.handle
        self.shape = (T, d_in, d_out, n)

    @property
    def ref(self):
        return ctypes.byref(self.c)


def marlaas_workspace_bytes(desc, want_bwd=False):
    return int(load().marlaas_workspace_bytes(desc.ref, 1 if want_bwd else 0))


def marlaas_u_stride(desc):
    return int(load().marlaas_u_stride(desc.ref))


def marlaas_set_workspace(ctx, tensor):
    """tensor: a CUDA tensor used as scratch (kept alive by the context object), or None."""
    ctx.workspace = tensor
    nbytes = tensor.numel() * tensor.element_size() if tensor is not None else 0
    _check(ctx, load().marlaas_set_workspace(ctx.handle, _ptr(tensor), nbytes))


def marlaas_lora_fwd(ctx, desc, y, u_save=None, stream=None):
    ldy = y.stride(0) if y.shape[0] > 0 else y.shape[1]
    _check(ctx, load().marlaas_lora_fwd(ctx.handle, desc.ref, _ptr(y), ldy, _ptr(u_save), _stream_ptr(stream)))


MARLAAS_STATIC_SCRATCH_BYTES = 32 << 20


def marlaas_packed_weight_bytes(d_in, d_out, direction=0):
    return int(load().marlaas_packed_weight_bytes(int(d_in), int(d_out), int(direction)))


def marlaas_pack_weight(ctx, W, layout, direction=0, stream=None):
    """A new uint8 CUDA tensor holding the packed copy of W (bf16; layout as in the descriptor)."""
    assert W.dtype == torch.bfloat16 and W.is_cuda
    d_in, d_out = (W.shape[0], W.shape[1]) if layout == MARLAAS_LAYOUT_MATH else (W.shape[1], W.shape[0])
    out = torch.empty(marlaas_packed_weight_bytes(d_in, d_out, direction), dtype=torch.uint8, device=W.device)
    _check(ctx, load().marlaas_pack_weight(ctx.handle, _ptr(W), W.stride(0), d_in, d_out, int(layout), int(direction),
                                           _ptr(out), _stream_ptr(stream)))
    return out


def marlaas_transpose_weight(ctx, W, layout, stream=None):
    """A new bf16 CUDA tensor holding the dense transposed copy of W (for the descriptor's W_t)."""
    assert W.dtype == torch.bfloat16 and W.is_cuda
    d_in, d_out = (W.shape[0], W.shape[1]) if layout == MARLAAS_LAYOUT_MATH else (W.shape[1], W.shape[0])
    out = torch.empty((W.shape[1], W.shape[0]), dtype=torch.bfloat16, device=W.device)
    _check(ctx, load().marlaas_transpose_weight(ctx.handle, _ptr(W), W.stride(0), d_in, d_out, int(layout), _ptr(out),
                                                _stream_ptr(stream)))
    return out


def marlaas_lora_fwd_static(ctx, desc, y, u_save=None, stream=None):
    ldy = y.stride(0) if y.shape[0] > 0 else y.shape[1]
    _check(ctx, load().marlaas_lora_fwd_static(ctx.handle, desc.ref, _ptr(y), ldy, _ptr(u_save), _stream_ptr(stream)))


def _desc_array(descs):
    arr = (marlaas_lora_desc * len(descs))()
    for i, d in enumerate(descs):
        arr[i] = d.c            # plain copy of the struct; the LoraDesc objects keep its host arrays alive
    return arr


def marlaas_workspace_bytes_multi(descs):
    return int(load().marlaas_workspace_bytes_multi(_desc_array(descs), len(descs)))


def marlaas_lora_fwd_multi(ctx, descs, ys, stream=None):
    """Forward of several projections of one input (same x, map, dtypes, layout): ys[p] receives projection p."""
    n = len(descs)
    yp = (ctypes.c_void_p * n)(*[y.data_ptr() for y in ys])
    ld = (ctypes.c_int64 * n)(*[(y.stride(0) if y.shape[0] > 0 else y.shape[1]) for y in ys])
    _check(ctx, load().marlaas_lora_fwd_multi(ctx.handle, _desc_array(descs), n, yp, ld, _stream_ptr(stream)))


def marlaas_lora_bwd(ctx, desc, dY, dX=None, dA=None, dB=None, u_saved=None, accumulate=False, stream=None):
    n = desc.shape[3]
    pa = pb = None
    if dA is MARLAAS_GRADS_IN_TABLE:
        pa = pb = MARLAAS_GRADS_IN_TABLE
    elif dA is not None:
        pa = (ctypes.c_void_p * max(n, 1))(*[t.data_ptr() for t in dA])
        pb = (ctypes.c_void_p * max(n, 1))(*[t.data_ptr() for t in dB])
    lddy = dY.stride(0) if dY.shape[0] > 0 else dY.shape[1]
    lddx = (dX.stride(0) if dX.shape[0] > 0 else dX.shape[1]) if dX is not None else 0
    _check(ctx, load().marlaas_lora_bwd(ctx.handle, desc.ref, _ptr(dY), lddy, _ptr(u_saved), _ptr(dX), lddx,
                                        pa, pb, 1 if accumulate else 0, _stream_ptr(stream)))


def marlaas_lora_bwd_adamw(ctx, desc, dY, states, hp, dX=None, u_saved=None, stream=None):
    """states: per adapter a dict of tensors master_A, master_B, m_A, v_A, m_B, v_B (fp32) and A_next,
    B_next (bf16); hp: dict lr, beta1, beta2, eps, weight_decay, step."""
    n = desc.shape[3]
    keys = [f[0] for f in marlaas_adapter_state._fields_]
    arr = (marlaas_adapter_state * max(n, 1))()
    for t, st in enumerate(states):
        for k in keys:
            setattr(arr[t], k, st[k].data_ptr())
    h = marlaas_adamw(hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"], int(hp["step"]))
    lddy = dY.stride(0) if dY.shape[0] > 0 else dY.shape[1]
    lddx = (dX.stride(0) if dX.shape[0] > 0 else dX.shape[1]) if dX is not None else 0
    _check(ctx, load().marlaas_lora_bwd_adamw(ctx.handle, desc.ref, _ptr(dY), lddy, _ptr(u_saved), _ptr(dX), lddx,
                                              arr, ctypes.byref(h), _stream_ptr(stream)))


def marlaas_profile_enable(ctx, on):
    _check(ctx, load().marlaas_profile_enable(ctx.handle, 1 if on else 0))


def marlaas_profile_read(ctx, kernel):
    """(total milliseconds, launches) of one kernel family since profiling was enabled."""
    ms, cnt = ctypes.c_double(0.0), ctypes.c_int64(0)
    _check(ctx, load().marlaas_profile_read(ctx.handle, int(kernel), ctypes.byref(ms), ctypes.byref(cnt)))
    return ms.value, cnt.value
