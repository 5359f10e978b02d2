"""Pins of the oracle's optimizer step (oracle_adamw_step), on the CPU, against things other than
itself: a two-step example worked by hand, closed forms that follow from the update rule
(constant gradient, zero gradient, both decay rates zero), the invariance of Adam's trajectory
to the scale of the gradients, element-wise independence, and torch's AdamW run in float64.
A dropped bias correction, a coupled instead of a decoupled decay, eps inside the square root,
or swapped moments each fail at least one of them."""
import json
import os

import numpy as np
import pytest
import torch

from oracle import lora_oracle as oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "adamw_hand_example.json")
HP = dict(lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.05)


def _run(p, grads, hp, m=None, v=None, first_step=1):
    m = np.zeros_like(p) if m is None else m
    v = np.zeros_like(p) if v is None else v
    for i, g in enumerate(grads):
        p, m, v = oracle.adamw_step(p, m, v, g, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"], first_step + i)
    return p, m, v


def test_hand_example():
    ex = json.load(open(GOLD))
    hp = {k: ex[k] for k in ("lr", "beta1", "beta2", "eps", "weight_decay")}
    p, m, v = np.array([ex["p0"]]), np.zeros(1), np.zeros(1)
    for i, g in enumerate(ex["g"]):
        p, m, v = _run(p, [np.array([g])], hp, m, v, first_step=i + 1)
        assert abs(p[0] - ex["p"][i]) <= 2e-15, (i, p[0])
        assert abs(m[0] - ex["m"][i]) <= 1e-16 and abs(v[0] - ex["v"][i]) <= 1e-18


def test_constant_gradient_without_decay_moves_by_the_same_amount_every_step():
    """With the same g at every step the bias-corrected moments are exactly g and g^2, so each
    step subtracts lr * g / (|g| + eps)."""
    rng = np.random.default_rng(0)
    p0, g = rng.normal(size=50), rng.normal(size=50)
    hp = dict(HP, weight_decay=0.0)
    n = 7
    p, _, _ = _run(p0, [g] * n, hp)
    want = p0 - n * hp["lr"] * g / (np.abs(g) + hp["eps"])
    assert np.max(np.abs(p - want)) <= 1e-13


def test_zero_gradient_only_decays():
    p0 = np.linspace(-2, 2, 9)
    n = 5
    p, m, v = _run(p0, [np.zeros(9)] * n, HP)
    assert np.max(np.abs(p - p0 * (1 - HP["lr"] * HP["weight_decay"]) ** n)) <= 1e-15
    assert not m.any() and not v.any()


def test_decay_is_decoupled_from_the_moments():
    """The decay term never enters m or v: with and without decay the moments are identical."""
    rng = np.random.default_rng(1)
    p0, gs = rng.normal(size=20), list(rng.normal(size=(4, 20)))
    _, m1, v1 = _run(p0, gs, HP)
    _, m2, v2 = _run(p0, gs, dict(HP, weight_decay=0.0))
    assert np.array_equal(m1, m2) and np.array_equal(v1, v2)


def test_trajectory_does_not_depend_on_the_gradient_scale_when_eps_is_zero():
    rng = np.random.default_rng(2)
    p0, gs = rng.normal(size=30), rng.normal(size=(6, 30))
    hp = dict(HP, eps=0.0)
    pa, _, _ = _run(p0, list(gs), hp)
    pb, _, _ = _run(p0, list(gs * 1024.0), hp)       # a power of two: every intermediate scales exactly
    assert np.max(np.abs(pa - pb)) <= 1e-15


def test_without_memory_it_is_a_normalised_gradient_step():
    """beta1 = beta2 = 0: m = g, v = g^2, both corrections 1."""
    rng = np.random.default_rng(3)
    p0, g = rng.normal(size=40), rng.normal(size=40)
    hp = dict(HP, beta1=0.0, beta2=0.0)
    p, m, v = _run(p0, [g], hp)
    want = p0 * (1 - hp["lr"] * hp["weight_decay"]) - hp["lr"] * g / (np.abs(g) + hp["eps"])
    assert np.max(np.abs(p - want)) <= 1e-15 and np.array_equal(m, g) and np.max(np.abs(v - g * g)) <= 1e-18


def test_elements_are_independent_and_shape_does_not_matter():
    rng = np.random.default_rng(4)
    p0, m0, v0, g = rng.normal(size=(4, 6, 5))
    v0 = np.abs(v0)
    perm = rng.permutation(30)
    a = oracle.adamw_step(p0, m0, v0, g, 3e-3, 0.8, 0.95, 1e-6, 0.1, 4)
    b = oracle.adamw_step(p0.ravel()[perm], m0.ravel()[perm], v0.ravel()[perm], g.ravel()[perm], 3e-3, 0.8, 0.95, 1e-6, 0.1, 4)
    for x, y in zip(a, b):
        assert x.shape == (6, 5) and np.array_equal(x.ravel()[perm], y)


@pytest.mark.parametrize("wd", [0.0, 0.1])
def test_against_torch_adamw_in_float64(wd):
    rng = np.random.default_rng(5)
    p0, gs = rng.normal(size=(3, 17)), rng.normal(size=(6, 3, 17))
    hp = dict(lr=2e-3, beta1=0.85, beta2=0.98, eps=1e-7, weight_decay=wd)
    p, m, v = _run(p0, list(gs), hp)
    tp = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([tp], lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"], weight_decay=wd)
    for g in gs:
        tp.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
    st = opt.state[tp]
    assert np.max(np.abs(p - tp.detach().numpy())) <= 1e-14
    assert np.max(np.abs(m - st["exp_avg"].numpy())) <= 1e-15 and np.max(np.abs(v - st["exp_avg_sq"].numpy())) <= 1e-15


def test_step_below_one_is_an_error():
    z = np.zeros(3)
    with pytest.raises(RuntimeError):
        oracle.adamw_step(z, z, z, z, 1e-3, 0.9, 0.999, 1e-8, 0.0, 0)
