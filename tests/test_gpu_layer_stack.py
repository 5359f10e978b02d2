"""A decode step through a stack of layers (harness/layer_stack.py) on the GPU, through the C ABI:
every projection call of every layer against the fp64 oracle applied to that call's actual input,
the whole chain against the oracle applied layer by layer from the same x (rounding to bf16 where
the stack does), and the step replayed as one HIP graph against the eager step.

Outputs are bf16 here (each call feeds the next), so a call is held to the error the oracle's own
values have after rounding to bf16 (that floor plus 5 %, and one unit in the last place at most);
the end of the chain norm-wise (1e-2), since one-unit rounding differences between the two
chains feed forward from call to call."""
import numpy as np
import pytest
import torch

from paper_2605_08527_amd import api
from harness import workloads as wl
from harness.layer_stack import DecodeStack
from helpers import check_bf16, to_host

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def _round_bf16(a):
    return wl.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def _oracle_call(oracle, x_bits, pr, stack, ids):
    return oracle.fwd(x_bits, _bits(pr.W), [_bits(a) for a in pr.A], [_bits(b) for b in pr.B],
                      np.asarray(stack.ranks, np.int32), np.asarray(stack.scales, np.float32), ids, layout=wl.TORCH)


def _silu(a):
    return a / (1.0 + np.exp(-a))


def _make(T=100, d=256, d_kv=64, d_ff=512, L=2, packed=True, seed=3):
    rng = np.random.default_rng(seed)
    ranks, scales = [8, 16, 8, 16], [2.0, 1.0, 0.5, 2.0]
    ids = rng.integers(-1, len(ranks), size=T).astype(np.int32)
    ctx = api.marlaas_create(0)
    stack = DecodeStack(api, torch, ctx, torch.from_numpy(ids).cuda(), T, d, d_kv, d_ff, L, ranks, scales, seed=seed, packed=packed)
    return stack, ids


@pytest.mark.parametrize("packed", [True, False], ids=["packed", "plain"])
def test_every_call_and_the_chain_match_the_oracle(oracle, packed):
    stack, ids = _make(packed=packed)
    stack.step()
    torch.cuda.synchronize()
    f64 = lambda bits: wl.bf16_bits_to_f32(bits).astype(np.float64)
    x_chain = _bits(stack.x0)                               # the oracle's own chain, bf16 bits between calls
    for li, lay in enumerate(stack.layers):
        b, (qkv, o, gate_up, down) = lay["buf"], lay["groups"]
        # every call against the oracle on the input the call really had
        for g in (qkv, o, gate_up, down):
            for pr, out in zip(g.projs, g.outs):
                check_bf16(to_host(out), _oracle_call(oracle, _bits(g.x), pr, stack, ids), "layer %d %s" % (li, g.name))
        # the chain
        q = _round_bf16(_oracle_call(oracle, x_chain, qkv.projs[0], stack, ids))
        oo = _round_bf16(_oracle_call(oracle, q, o.projs[0], stack, ids))
        h = _round_bf16(f64(x_chain) + f64(oo))
        gg = _round_bf16(_oracle_call(oracle, h, gate_up.projs[0], stack, ids))
        up = _round_bf16(_oracle_call(oracle, h, gate_up.projs[1], stack, ids))
        m = _round_bf16(f64(_round_bf16(_silu(f64(gg)))) * f64(up))
        dn = _round_bf16(_oracle_call(oracle, m, down.projs[0], stack, ids))
        x_chain = _round_bf16(f64(h) + f64(dn))
    # The two chains round to bf16 after every call; where the fp32 and the fp64 sum fall on
    # different sides of a rounding boundary (about one element in a thousand per call) the next
    # call's input differs by one unit in the last place, which moves a few per cent of its
    # outputs across a boundary in turn.  So the end of the chain is compared norm-wise and on
    # the mean, and most elements must still be the same bf16 value.
    got, ref = to_host(stack.out), f64(x_chain)
    mx, mean, nrm = wl.rel_err_stats(got, ref)
    assert np.all(np.isfinite(got))
    assert nrm <= 1e-2 and mean <= 2e-3, "end of the chain: max %.3e mean %.3e norm-wise %.3e" % (mx, mean, nrm)
    assert np.mean(got != ref) < 0.5


def test_graph_replay_of_the_stack_matches_the_eager_step():
    """Captured on its first call (the passes allocate nothing), replayed several times with eager
    work and synchronisation between the replays: every replay bit-equal to the eager step."""
    stack, _ = _make(T=64, L=3, seed=5)
    graph = stack.capture()
    graph.replay()
    torch.cuda.synchronize()
    first = _bits(stack.out).copy()
    stack.step()
    torch.cuda.synchronize()
    eager = _bits(stack.out).copy()
    assert np.array_equal(first, eager)
    for rep in range(3):
        stack.out.fill_(float("nan"))
        stack.layers[0]["buf"]["q"].fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(_bits(stack.out), eager), "replay %d" % rep
