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


# ---------------------------------------------------------------- momentum and weight decay
def test_momentum_closed_form_with_constant_sign_update():
    """Same rank-one G every step, no parameter scaling: v stays G*G, U = sign(G) and the scaled
    update D = lr sign(G) is constant, so m_t = (1 - beta1^t) D and
    W_t = W_0 - lr sign(G) sum_{s<=t} (1 - beta1^s)."""
    rng = np.random.default_rng(3)
    g = np.outer(rng.uniform(0.5, 2, 6) * rng.choice([-1, 1], 6), rng.uniform(0.5, 2, 4))
    w0 = rng.standard_normal((6, 4))
    beta1, lr = 0.9, 0.02
    w, st = w0, O.adafactor_zero_state(6, 4, True, momentum=True)
    acc = 0.0
    for t in range(1, 6):
        w, st = O.adafactor_step(w, g, st, step=t, lr=lr, factored=True, scale_by_param=False, beta1=beta1)
        acc += 1.0 - beta1 ** t
        np.testing.assert_allclose(st["m"], (1.0 - beta1 ** t) * lr * np.sign(g), rtol=1e-10)
        np.testing.assert_allclose(w, w0 - lr * np.sign(g) * acc, rtol=1e-10, atol=1e-13)


def test_variants_reduce_to_the_plain_update():
    p, g = SI.make_adafactor_case(9, 12, seed=3)
    base, _ = O.adafactor_step(p, g, O.adafactor_zero_state(9, 12, True), step=1, lr=0.01, factored=True)
    same, st = O.adafactor_step(p, g, O.adafactor_zero_state(9, 12, True), step=1, lr=0.01, factored=True,
                                beta1=0.0, weight_decay=0.0)
    assert np.array_equal(base, same) and "m" not in st
    # beta1 -> 0+ : m = D, same parameters
    near, st = O.adafactor_step(p, g, O.adafactor_zero_state(9, 12, True, momentum=True), step=1, lr=0.01,
                                factored=True, beta1=1e-12)
    np.testing.assert_allclose(near, base, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(st["m"], p - base, rtol=1e-9, atol=1e-14)


def test_weight_decay_is_decoupled():
    """The decay term is lr * wd * W whatever the gradient does: it adds to the plain update, and with
    the parameter-scale factor switched off a vanishing gradient leaves exactly W (1 - lr wd)."""
    p, g = SI.make_adafactor_case(8, 10, seed=4)
    lr, wd = 0.05, 0.1
    plain, _ = O.adafactor_step(p, g, O.adafactor_zero_state(8, 10, False), step=1, lr=lr, factored=False)
    dec, _ = O.adafactor_step(p, g, O.adafactor_zero_state(8, 10, False), step=1, lr=lr, factored=False,
                              weight_decay=wd)
    np.testing.assert_allclose(dec, plain - lr * wd * p, rtol=1e-13, atol=1e-15)
    zero_g, _ = O.adafactor_step(p, np.zeros_like(g), O.adafactor_zero_state(8, 10, False), step=1, lr=lr,
                                 factored=False, weight_decay=wd, scale_by_param=False)
    np.testing.assert_allclose(zero_g, p * (1 - lr * wd), rtol=1e-13)
    # momentum does not touch the decay term: it acts on D only
    both, st = O.adafactor_step(p, g, O.adafactor_zero_state(8, 10, False, momentum=True), step=1, lr=lr,
                                factored=False, weight_decay=wd, beta1=0.5)
    np.testing.assert_allclose(both, p - 0.5 * (p - plain) - lr * wd * p, rtol=1e-12, atol=1e-15)


def test_weight_decay_against_torch_library_adafactor():
    """torch.optim.Adafactor applies decoupled decay as W (1 - lr_t wd) with its own step size lr_t; fed
    the same lr_t the oracle's update agrees over three steps (unfactored and factored)."""
    if not hasattr(torch.optim, "Adafactor"):
        pytest.skip("torch.optim.Adafactor not available")
    for rows, cols in ((6, 9), (1, 12)):
        p0, _ = SI.make_adafactor_case(rows, cols, seed=6)
        tp = torch.nn.Parameter(torch.from_numpy(p0.copy()).reshape(rows, cols) if rows > 1
                                else torch.from_numpy(p0.copy()).reshape(cols))
        opt = torch.optim.Adafactor([tp], lr=0.01, beta2_decay=-0.8, eps=(1e-30, 1e-3), d=1.0, weight_decay=0.2,
                                    foreach=False)
        fact = rows > 1
        w, st = p0, O.adafactor_zero_state(rows, cols, fact)
        for t in (1, 2, 3):
            _, g = SI.make_adafactor_case(rows, cols, seed=60 + t, grad_std=1e-2 * t)
            tp.grad = torch.from_numpy(g.copy()).reshape(tp.shape)
            opt.step()
            # torch's relative step: min(lr, 1/sqrt(t)), and its parameter scale multiplies the update only
            lr_t = min(0.01, 1.0 / math.sqrt(t))
            w, st = O.adafactor_step(w, g, st, step=t, lr=lr_t, factored=fact, weight_decay=0.2)
            np.testing.assert_allclose(w.reshape(tp.shape), tp.detach().numpy(), rtol=1e-9, atol=1e-12)
