"""marlaas_lora_bwd_adamw on the GPU, through the C ABI, against the fp64 oracle: the backward of
the oracle followed by the oracle's AdamW step on every factor, from the same inputs and the same
optimizer state (fp32 values widened exactly).

What is compared and how: dX at the backward's tolerance (floored relative error max 1e-2, mean
1e-3); the new fp32 master values through the update they received, in units of the learning
rate, |p_gpu - p_oracle| <= 1e-3 lr + 1e-6 |p| (the update is m_hat / (sqrt(v_hat) + eps), O(1),
and inherits the gradient's fp32 summation error); the new moments at the gradients' tolerance;
the bf16 factors of the next version bit for bit against the library's own master values rounded
to nearest even (the decision is taken in the kernel's precision on both sides)."""
import numpy as np
import pytest
import torch

from paper_2605_08527_amd import api
from harness import workloads as wl
from helpers import HipLayer, assert_close, oracle_grads_in_layout, to_dev, to_host

pytestmark = pytest.mark.gpu
HP = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.1)


def _state(w, rng, zero=False):
    """Optimizer state as numpy arrays per adapter: fp32 masters equal to the bf16 factors, moments
    as after a few updates (or zero)."""
    st = []
    for A, B in zip(w["A"], w["B"]):
        e = {}
        for k, f in (("A", A), ("B", B)):
            e["master_" + k] = wl.bf16_bits_to_f32(f).astype(np.float32)
            g_rms = 30.0       # order of magnitude of the gradients of these workloads
            e["m_" + k] = (np.zeros(f.shape) if zero else rng.normal(0, 0.3 * g_rms, size=f.shape)).astype(np.float32)
            e["v_" + k] = (np.zeros(f.shape) if zero else rng.uniform(0.5, 1.5, size=f.shape) * g_rms ** 2).astype(np.float32)
        st.append(e)
    return st


def _dev_state(st, L, in_place):
    out = []
    for t, e in enumerate(st):
        d = {k: torch.from_numpy(v.copy()).cuda() for k, v in e.items()}
        d["A_next"] = L.A[t] if in_place else torch.zeros_like(L.A[t])
        d["B_next"] = L.B[t] if in_place else torch.zeros_like(L.B[t])
        out.append(d)
    return out


def _oracle_step(oracle, w, st, hp):
    args = (w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"])
    dX, dA, dB = oracle.bwd(*args, w["dY"], layout=w["layout"])
    dA, dB = oracle_grads_in_layout(dA, dB, w["layout"])
    new = []
    for t, e in enumerate(st):
        n = {}
        for k, g in (("A", dA[t]), ("B", dB[t])):
            p, m, v = oracle.adamw_step(e["master_" + k].astype(np.float64), e["m_" + k].astype(np.float64),
                                        e["v_" + k].astype(np.float64), np.ascontiguousarray(g), hp["lr"], hp["beta1"],
                                        hp["beta2"], hp["eps"], hp["weight_decay"], hp["step"])
            n["master_" + k], n["m_" + k], n["v_" + k], n["g_" + k] = p, m, v, np.asarray(g)
        new.append(n)
    return dX, new


def _check_state(dev, ref, old, hp, tag, only=None):
    for k in ("A", "B"):
        p = dev["master_" + k].cpu().numpy().astype(np.float64)
        want = ref["master_" + k]
        sel = np.ones(p.shape, bool) if only is None else only[k]
        bound = 1e-3 * hp["lr"] + 1e-6 * np.abs(want)
        assert np.all(np.abs(p - want)[sel] <= bound[sel]), "%s master_%s: worst %.3e lr" % (
            tag, k, np.max((np.abs(p - want) / hp["lr"])[sel]))
        assert np.any(p != old["master_" + k]), tag + ": the master copy did not move"
        assert_close(dev["m_" + k].cpu().numpy().astype(np.float64), ref["m_" + k], tag + " m_" + k)
        assert_close(dev["v_" + k].cpu().numpy().astype(np.float64), ref["v_" + k], tag + " v_" + k)
        bits = dev[k + "_next"].view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(bits, wl.f32_to_bf16_bits(dev["master_" + k].cpu().numpy())), tag + " next " + k


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("table", [False, True], ids=["lists", "table"])
def test_single_task_training_step_twice_in_place(oracle, layout, table):
    """The paper's training regime: every token of the batch belongs to the one task being trained
    (identity map, long segment: the reductions split the tokens over workgroups).  Two updates in
    a row on the same buffers, the second reading the factors the first wrote."""
    rng = np.random.default_rng(11 + layout)
    T, K, N, r = 4096, 1024, 512, 32
    w = wl.make_layer(21 + layout, T, K, N, [r], [2.0], np.zeros(T, np.int32), dtype="bf16", layout=layout, want_dY=True)
    L = HipLayer(w, want_bwd=True, table=table)
    st = _state(w, rng)
    dev = _dev_state(st, L, in_place=True)
    for step in (5, 6):
        hp = dict(HP, step=step)
        y, u = L.fwd(save_u=True)
        dX = torch.full((T, K), float("nan"), dtype=torch.float32, device="cuda")
        api.marlaas_lora_bwd_adamw(L.ctx, L.desc, L.dY, dev, hp, dX=dX, u_saved=u)
        torch.cuda.synchronize()
        dX_ref, new = _oracle_step(oracle, w, st, hp)
        assert_close(to_host(dX), dX_ref, "dX step %d" % step)
        _check_state(dev[0], new[0], st[0], hp, "step %d" % step)
        # the oracle's own next version: its state, its factors rounded to bf16, a fresh dY
        st = [{k: v.astype(np.float32) for k, v in new[0].items() if not k.startswith("g_")}]
        w["A"] = [wl.f32_to_bf16_bits(new[0]["master_A"].astype(np.float32))]
        w["B"] = [wl.f32_to_bf16_bits(new[0]["master_B"].astype(np.float32))]
        w["dY"] = wl.f32_to_bf16_bits(rng.normal(size=(T, N)).astype(np.float32))
        L.dY.copy_(to_dev(w["dY"]))
        # (the library keeps its own fp32 state; the oracle's is the oracle's: they stay within tolerance)


@pytest.mark.parametrize("layout", [0, 1])
def test_several_adapters_short_segments_next_version_committed_by_hot_swap(oracle, layout):
    """Three adapters of different ranks plus one without tokens, tokens interleaved and some without
    adapter: separate buffers receive the next version, the served version is untouched, the
    adapter without tokens keeps its state bit for bit; committing the next version into the
    adapter table makes the forward use it."""
    rng = np.random.default_rng(31 + layout)
    T, K, N = 1500, 520, 328
    ranks, scales = [8, 16, 32, 16], [2.0, 0.5, 1.0, 2.0]
    ids = rng.integers(-1, 3, size=T).astype(np.int32)           # adapter 3 has no tokens
    w = wl.make_layer(41 + layout, T, K, N, ranks, scales, ids, dtype="bf16", layout=layout, want_dY=True)
    L = HipLayer(w, want_bwd=True, table=True)
    st = _state(w, rng)
    dev = _dev_state(st, L, in_place=False)
    served = [(a.clone(), b.clone()) for a, b in zip(L.A, L.B)]
    hp = dict(HP, step=3)
    dX = torch.full((T, K), float("nan"), dtype=torch.float32, device="cuda")
    api.marlaas_lora_bwd_adamw(L.ctx, L.desc, L.dY, dev, hp, dX=dX)        # u recomputed
    torch.cuda.synchronize()
    dX_ref, new = _oracle_step(oracle, w, st, hp)
    assert_close(to_host(dX), dX_ref, "dX")
    for t in range(3):
        _check_state(dev[t], new[t], st[t], hp, "adapter %d" % t)
        assert torch.equal(L.A[t], served[t][0]) and torch.equal(L.B[t], served[t][1])
    for k, v in st[3].items():
        assert np.array_equal(dev[3][k].cpu().numpy(), v), "adapter without tokens: " + k
    assert not dev[3]["A_next"].any() and not dev[3]["B_next"].any()
    # commit version v + 1 of the trained adapters and serve it
    for t in range(3):
        api.marlaas_adapter_table_update(L.ctx, L.table, 0, t, dev[t]["A_next"], dev[t]["B_next"], ranks[t], scales[t])
    y, _ = L.fwd()
    w2 = dict(w)
    w2["A"] = [wl.f32_to_bf16_bits(new[t]["master_A"].astype(np.float32)) for t in range(3)] + [w["A"][3]]
    w2["B"] = [wl.f32_to_bf16_bits(new[t]["master_B"].astype(np.float32)) for t in range(3)] + [w["B"][3]]
    y_ref = oracle.fwd(w2["x"], w2["W"], w2["A"], w2["B"], w2["ranks"], w2["scales"], w2["ids"], layout=layout)
    assert_close(to_host(y), y_ref, "forward on the committed version")


def test_first_update_from_zero_state(oracle):
    """m = v = 0, step 1: the update is lr g / (|g| + eps), a sign; where the gradient is within its
    own summation error of zero either sign is a correct result, so those elements are left out."""
    rng = np.random.default_rng(51)
    T, K, N, r = 2048, 512, 256, 16
    w = wl.make_layer(61, T, K, N, [r], [2.0], np.zeros(T, np.int32), dtype="bf16", layout=1, want_dY=True)
    L = HipLayer(w, want_bwd=True)
    st = _state(w, rng, zero=True)
    dev = _dev_state(st, L, in_place=False)
    hp = dict(HP, step=1)
    api.marlaas_lora_bwd_adamw(L.ctx, L.desc, L.dY, dev, hp)
    torch.cuda.synchronize()
    _, new = _oracle_step(oracle, w, st, hp)
    only = {k: np.abs(new[0]["g_" + k]) > 1e-3 * np.sqrt(np.mean(new[0]["g_" + k] ** 2)) for k in ("A", "B")}
    assert all(v.mean() > 0.99 for v in only.values())
    _check_state(dev[0], new[0], st[0], hp, "first step", only=only)


def test_error_paths():
    rng = np.random.default_rng(71)
    T, K, N = 64, 64, 64
    w = wl.make_layer(81, T, K, N, [8] * 9, [1.0] * 9, rng.integers(0, 9, size=T).astype(np.int32), dtype="bf16",
                      layout=0, want_dY=True)
    L = HipLayer(w, want_bwd=True)
    dev = _dev_state(_state(w, rng), L, in_place=False)
    with pytest.raises(api.MarlaasError) as e:
        api.marlaas_lora_bwd_adamw(L.ctx, L.desc, L.dY, dev, dict(HP, step=1))
    assert e.value.status == -6     # MARLAAS_EUNSUPPORTED
    w = wl.make_layer(82, T, K, N, [8], [1.0], np.zeros(T, np.int32), dtype="bf16", layout=0, want_dY=True)
    L = HipLayer(w, want_bwd=True)
    dev = _dev_state(_state(w, rng), L, in_place=False)
    with pytest.raises(api.MarlaasError) as e:
        api.marlaas_lora_bwd_adamw(L.ctx, L.desc, L.dY, dev, dict(HP, step=0))
    assert e.value.status == -1     # MARLAAS_EINVAL
