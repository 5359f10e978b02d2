"""marlaas_lora_fwd_static (the forward for callers that cannot allocate: its scratch is a static
array in the library's device code) against marlaas_lora_fwd on the same inputs, through the C ABI:
two calls in a row on one GPU, the second with a smaller input, each compared with the existing
entry point (floored relative error max <= 1e-2, mean <= 1e-3; these paths are deterministic, so
the results are in fact bit-identical) and with the fp64 oracle; then the size limit."""
import numpy as np
import pytest
import torch

from paper_2605_08527_amd import api
from harness import workloads as wl
from helpers import HipLayer, assert_close, to_host

pytestmark = pytest.mark.gpu


def _both(oracle, w, table, tag):
    L = HipLayer(w, table=table)
    y_ref, u_ref = L.fwd(save_u=True)                      # existing entry point, caller's workspace
    api.marlaas_set_workspace(L.ctx, None)                 # the static variant must not need it
    y = torch.full((L.T, L.N), float("nan"), dtype=torch.float32, device="cuda")
    u = torch.zeros((L.T, api.marlaas_u_stride(L.desc)), dtype=torch.float32, device="cuda")
    api.marlaas_lora_fwd_static(L.ctx, L.desc, y, u_save=u)
    torch.cuda.synchronize()
    assert_close(to_host(y), to_host(y_ref), tag + " y vs marlaas_lora_fwd")
    assert_close(to_host(u), to_host(u_ref), tag + " u vs marlaas_lora_fwd")
    assert torch.equal(y, y_ref) and torch.equal(u, u_ref), tag + ": not bit-identical to marlaas_lora_fwd"
    ref = oracle.fwd(w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"], layout=w["layout"])
    assert_close(to_host(y), ref, tag + " y vs oracle")
    return L


@pytest.mark.parametrize("table", [False, True], ids=["lists", "table"])
def test_static_scratch_forward_twice_then_limit(oracle, table):
    rng = np.random.default_rng(77)
    # first call: decode-sized (split contraction, fused shrink: partial sums, u and tables in scratch)
    T1, ranks = 256, [16, 8, 32, 16, 24]
    ids1 = rng.integers(-1, len(ranks), size=T1).astype(np.int32)
    w1 = wl.make_layer(201, T1, 1024, 1536, ranks, [2.0, 1.0, 0.5, 2.0, 1.0], ids1, dtype="bf16", layout=wl.TORCH)
    keep = _both(oracle, w1, table, "first")
    # second call, smaller input, other layout: whatever the first call left in the array must not matter
    T2 = 72
    ids2 = rng.integers(-1, 3, size=T2).astype(np.int32)
    w2 = wl.make_layer(202, T2, 520, 384, [8, 16, 24], [1.0, 2.0, 0.5], ids2, dtype="bf16", layout=wl.MATH)
    _both(oracle, w2, table, "second")
    # a forward that needs more scratch than the array holds is refused, with a message
    T3 = 2048
    ids3 = rng.integers(0, 2, size=T3).astype(np.int32)
    w3 = wl.make_layer(203, T3, 4096, 4096, [16, 16], [2.0, 2.0], ids3, dtype="bf16", layout=wl.TORCH)
    L3 = HipLayer(w3, table=table)
    need = api.marlaas_workspace_bytes(L3.desc, False)
    assert need > api.MARLAAS_STATIC_SCRATCH_BYTES, "test shape no longer exceeds the static scratch (%d bytes)" % need
    y3 = torch.empty((T3, 4096), dtype=torch.float32, device="cuda")
    with pytest.raises(api.MarlaasError) as e:
        api.marlaas_lora_fwd_static(L3.ctx, L3.desc, y3)
    assert e.value.status == -4 and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    del keep
