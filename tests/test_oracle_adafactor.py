"""Pins for the oracle's Adafactor step (CPU only): closed forms, invariants and torch's
library optimizer."""
import math

import numpy as np
import pytest
import torch

import synth_inputs as SI
from oracle import t5_oracle as O


def test_beta2_schedule():
    assert O.adafactor_beta2(1, 0.8) == 0.0
    assert abs(O.adafactor_beta2(2, 0.8) - 0.42565) < 5e-6
    assert abs(O.adafactor_beta2(3, 0.8) - 0.58476) < 5e-6


def test_rank_one_gradient_first_step_is_sign_descent():
    """t = 1, G = a b^T: the factored estimate equals G*G exactly, so U = sign(G), RMS(U) = 1 (no
    clipping) and W' = W - lr * max(eps2, RMS(W)) * sign(G)."""
    rng = np.random.default_rng(0)
    a = rng.uniform(0.5, 2.0, 7) * rng.choice([-1, 1], 7)
    b = rng.uniform(0.5, 2.0, 5) * rng.choice([-1, 1], 5)
    g = np.outer(a, b)
    w = rng.standard_normal((7, 5))
    st = O.adafactor_zero_state(7, 5, True)
    w1, st1 = O.adafactor_step(w, g, st, step=1, lr=0.01, factored=True)
    alpha = 0.01 * max(1e-3, math.sqrt(np.mean(w * w)))
    np.testing.assert_allclose(w1, w - alpha * np.sign(g), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(st1["vr"], a * a * np.mean(b * b), rtol=1e-12)
    np.testing.assert_allclose(st1["vc"], b * b * np.mean(a * a), rtol=1e-12)
    # factored == unfactored when G*G has rank one
    w2, _ = O.adafactor_step(w, g, O.adafactor_zero_state(7, 5, False), step=1, lr=0.01, factored=False)
    np.testing.assert_allclose(w2, w1, rtol=1e-12, atol=1e-14)
    # gradient scale does not matter at t = 1
    w3, _ = O.adafactor_step(w, 37.0 * g, st, step=1, lr=0.01, factored=True)
    np.testing.assert_allclose(w3, w1, rtol=1e-12, atol=1e-14)


def test_small_parameter_uses_eps2_and_scale_by_param_off():
    g = np.outer([1.0, -2.0], [3.0, 1.0, -1.0])
    w = np.full((2, 3), 1e-6)
    w1, _ = O.adafactor_step(w, g, O.adafactor_zero_state(2, 3, True), step=1, lr=0.5, factored=True)
    np.testing.assert_allclose(w1, w - 0.5 * 1e-3 * np.sign(g), rtol=1e-12)
    w2, _ = O.adafactor_step(w, g, O.adafactor_zero_state(2, 3, True), step=1, lr=0.5, factored=True,
                             scale_by_param=False)
    np.testing.assert_allclose(w2, w - 0.5 * np.sign(g), rtol=1e-12)


def test_update_clipping_bounds_rms():
    """At t >= 2 with a gradient much larger than the history, RMS(U) > 1 and is clipped to 1."""
    p, g = SI.make_adafactor_case(24, 40, seed=1)
    st = O.adafactor_zero_state(24, 40, True)
    p1, st = O.adafactor_step(p, g, st, step=1, lr=0.01, factored=True)
    big = 50.0 * g
    p2, st2 = O.adafactor_step(p1, big, st, step=2, lr=0.01, factored=True, scale_by_param=False)
    applied = (p1 - p2) / 0.01
    assert abs(math.sqrt(np.mean(applied ** 2)) - 1.0) < 1e-9
    # unclipped magnitude would have been larger
    p3, _ = O.adafactor_step(p1, big, st, step=2, lr=0.01, factored=True, scale_by_param=False, clip=1e9)
    assert math.sqrt(np.mean(((p1 - p3) / 0.01) ** 2)) > 1.2
    # invariant: mean(vr) == mean(vc) from a zero state
    np.testing.assert_allclose(st2["vr"].mean(), st2["vc"].mean(), rtol=1e-12)


@pytest.mark.skipif(not hasattr(torch.optim, "Adafactor"), reason="torch build has no Adafactor")
@pytest.mark.parametrize("rows,cols", [(24, 40), (1, 33)])
def test_three_steps_against_torch_library_adafactor(rows, cols):
    """torch.optim.Adafactor (float64) implements the same rule when lr < 1/sqrt(t); a 2-D tensor
    is factored, a 1-D tensor is not."""
    factored = rows > 1
    p, _ = SI.make_adafactor_case(rows, cols, seed=2)
    tp = torch.nn.Parameter(torch.from_numpy(p.copy() if factored else p[0].copy()))
    opt = torch.optim.Adafactor([tp], lr=0.01, beta2_decay=-0.8, eps=(1e-30, 1e-3), d=1.0,
                                weight_decay=0.0, foreach=False)
    st = O.adafactor_zero_state(rows, cols, factored)
    w = p
    for t in (1, 2, 3):
        _, g = SI.make_adafactor_case(rows, cols, seed=10 + t, grad_std=1e-2 * t * t)
        tp.grad = torch.from_numpy(g.copy() if factored else g[0].copy())
        opt.step()
        w, st = O.adafactor_step(w, g, st, step=t, lr=0.01, factored=factored)
        ref = tp.detach().numpy().reshape(rows, cols)
        np.testing.assert_allclose(w, ref, rtol=1e-10, atol=1e-13)


def test_resume_is_bit_identical():
    p, _ = SI.make_adafactor_case(16, 12, seed=3)
    grads = [SI.make_adafactor_case(16, 12, seed=20 + t)[1] for t in range(3)]
    w, st = p, O.adafactor_zero_state(16, 12, True)
    for t, g in enumerate(grads, 1):
        w, st = O.adafactor_step(w, g, st, step=t, lr=0.01, factored=True)
    w2, st2 = p, O.adafactor_zero_state(16, 12, True)
    for t, g in enumerate(grads[:2], 1):
        w2, st2 = O.adafactor_step(w2, g, st2, step=t, lr=0.01, factored=True)
    w2c, st2c = w2.copy(), {k: v.copy() for k, v in st2.items()}
    w3, _ = O.adafactor_step(w2c, grads[2], st2c, step=3, lr=0.01, factored=True)
    assert np.array_equal(w3, w)
