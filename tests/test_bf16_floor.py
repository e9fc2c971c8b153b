"""CPU checks of the bf16 error-floor model (tests/bf16_model.py) that the GPU tolerances are derived from.

1. Structure: with the rounding switched off the model must BE the oracle (block and decoder layer, every
   feed-forward variant, with and without dropout) -- so the only thing it adds is the list of rounded tensors.
2. Values: the floors at the T5.1.1-Small block shape, both readings of the logit scale and both
   split-operand variants of the score path, against tests/golden/bf16_floor_c2_small.json
   (written by tests/golden/make_bf16_floor.py), and what they imply for the stated 2e-2 / 2e-3 target.
3. The rule that turns a floor into a bound.
"""
import json
import os
from dataclasses import replace

import numpy as np
import pytest

import bf16_model as M
import synth_inputs as SI
from oracle import t5_oracle as O
from parity_util import MARGIN, STATED_BF16, max_margin, mean_margin, tol_from_floor

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "bf16_floor_c2_small.json")

SMALL = SI.BlockConfig("floor_small", 90, batch=2, seq=48, d_model=64, n_heads=2, d_kv=16, d_ff=96, attn_scale=0.25)
VARIANTS = [
    SMALL,
    replace(SMALL, name="floor_causal", causal=True),
    replace(SMALL, name="floor_relu", mlp="relu"),
    replace(SMALL, name="floor_erf", mlp="geglu_erf", causal=True),
    replace(SMALL, name="floor_drop", dropout_rate=float(np.float32(0.1)), dropout_seed=77),
    replace(SMALL, name="floor_drop_relu", mlp="relu", causal=True, dropout_rate=float(np.float32(0.25)), dropout_seed=5),
]


def _case(cfg):
    w = SI.make_weights(cfg)
    w.update(SI.make_random_scales(cfg))
    x, dy = SI.make_activations(cfg)
    return w, x, dy


@pytest.mark.parametrize("cfg", VARIANTS, ids=[c.name for c in VARIANTS])
def test_model_without_rounding_is_the_oracle(cfg, monkeypatch):
    monkeypatch.setattr(M, "rb", lambda a: np.asarray(a, dtype=np.float64))
    w, x, dy = _case(cfg)
    y, saved = O.block_fwd(cfg, x, w)
    dx, g = O.block_bwd(cfg, dy, w, saved)
    my, mdx, mg = M.block_model(cfg, x, w, dy)
    assert set(mg) == set(g)
    np.testing.assert_allclose(my, y, rtol=0, atol=1e-11)
    np.testing.assert_allclose(mdx, dx, rtol=0, atol=1e-10)
    for k in g:
        np.testing.assert_allclose(mg[k], g[k], rtol=0, atol=1e-9 * max(1.0, np.abs(g[k]).max()), err_msg=k)
    # the split-operand variants change nothing either once nothing is rounded
    sy, sdx, _ = M.block_model(cfg, x, w, dy, split_qk=True, split_n1=True)
    np.testing.assert_allclose(sy, y, rtol=0, atol=1e-11)
    np.testing.assert_allclose(sdx, dx, rtol=0, atol=1e-10)


@pytest.mark.parametrize("cfg", [replace(c, enc_seq=37, causal=True) for c in (VARIANTS[0], VARIANTS[2], VARIANTS[4])],
                         ids=["dec", "dec_relu", "dec_drop"])
def test_decoder_model_without_rounding_is_the_oracle(cfg, monkeypatch):
    monkeypatch.setattr(M, "rb", lambda a: np.asarray(a, dtype=np.float64))
    w, x, dy = _case(cfg)
    enc = SI.make_encoder_output(cfg)
    y, saved = O.decoder_block_fwd(cfg, x, enc, w)
    dx, denc, g = O.decoder_block_bwd(cfg, dy, w, saved)
    my, mdx, mde, mg = M.decoder_block_model(cfg, x, enc, w, dy)
    assert set(mg) == set(g)
    np.testing.assert_allclose(my, y, rtol=0, atol=1e-11)
    np.testing.assert_allclose(mdx, dx, rtol=0, atol=1e-10)
    np.testing.assert_allclose(mde, denc, rtol=0, atol=1e-10)
    for k in g:
        np.testing.assert_allclose(mg[k], g[k], rtol=0, atol=1e-9 * max(1.0, np.abs(g[k]).max()), err_msg=k)


def _max_diff(a, b):
    if isinstance(a, dict):
        return max(_max_diff(a[k], b[k]) for k in b)
    if isinstance(a, list):
        return max(_max_diff(x, y) for x, y in zip(a, b))
    return float(np.abs(np.asarray(a) - np.asarray(b)).max())


@pytest.mark.parametrize("tied,rate", [(False, 0.0), (True, 0.0), (False, 0.2), (True, 0.2)])
def test_stack_models_without_rounding_are_the_oracle(tied, rate, monkeypatch):
    monkeypatch.setattr(M, "rb", lambda a: np.asarray(a, dtype=np.float64))
    blk = SI.BlockConfig("floor_stack", 95, batch=2, seq=24, d_model=32, n_heads=2, d_kv=8, d_ff=48, causal=True,
                         attn_scale=0.3, dropout_rate=float(np.float32(rate)), dropout_seed=7)
    sc = SI.StackConfig("floor_stack", blk, n_layers=2, vocab=37, tied_logits=tied, z_loss=1e-2)
    w = SI.make_stack_weights(sc)
    SI.make_stack_random_scales(sc, w)
    tokens, targets = SI.make_tokens(sc, ignore_fraction=0.2)
    loss, saved = O.stack_loss(sc, tokens, targets, w)
    g = O.stack_loss_grad(sc, w, saved)
    ml, mg = M.stack_model(sc, tokens, targets, w)
    assert abs(ml - loss) <= 1e-12 and _max_diff(mg, g) <= 1e-12
    ec = SI._encdec("floor_ec", 96, 2, 20, 12, 32, 2, 8, 48, 2, 2, 37, z_loss=1e-2, block=dict(dtype="f32"))
    ec = replace(ec, tied_logits=tied,
                 enc_block=replace(ec.enc_block, dropout_rate=float(np.float32(rate)), dropout_seed=3),
                 dec_block=replace(ec.dec_block, dropout_rate=float(np.float32(rate)), dropout_seed=4))
    w = SI.make_encdec_weights(ec)
    SI.make_encdec_random_scales(ec, w)
    et, dt, tg = SI.make_encdec_tokens(ec, ignore_fraction=0.15)
    loss, saved = O.encdec_loss(ec, et, dt, tg, w)
    g = O.encdec_loss_grad(ec, w, saved)
    ml, mg = M.encdec_model(ec, et, dt, tg, w)
    assert abs(ml - loss) <= 1e-12 and _max_diff(mg, g) <= 1e-12


def test_rounding_is_bf16_round_to_nearest_even():
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: goes to the even mantissa (1); 1 + 3 * 2^-8 goes up to 1 + 2^-6
    a = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 3 * 2.0 ** -8, -3.0, 1e-30])
    r = M.rb(a)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 + 2.0 ** -7 and r[3] == 1.0 + 2.0 ** -6 and r[4] == -3.0
    assert abs(r[5] / 1e-30 - 1.0) <= 2.0 ** -8
    x = np.random.default_rng(0).standard_normal(10000)
    rel = np.abs(M.rb(x) - x) / np.abs(x)
    assert rel.max() <= 2.0 ** -8 and 0.8e-3 < rel.mean() < 1.6e-3     # half an ulp at most; about 2^-8 * 0.36 mean


@pytest.fixture(scope="module")
def floors():
    from golden.make_bf16_floor import floors as compute
    return compute()


def test_floors_match_golden(floors):
    with open(GOLDEN) as fh:
        gold = json.load(fh)
    assert set(gold) == set(floors)
    for key in gold:
        for name, (gmax, gmean) in gold[key].items():
            fmax, fmean = floors[key][name]
            # same seeds, same arithmetic: differences come from the BLAS summation order only
            assert abs(fmean - gmean) <= 0.02 * gmean, (key, name, fmean, gmean)
            assert abs(fmax - gmax) <= 0.25 * gmax, (key, name, fmax, gmax)


def test_what_the_floors_say_about_the_stated_target(floors):
    sc, lit = floors["scaled/plain"], floors["literal/plain"]
    grads = [k for k in sc if k not in ("y", "dx")]
    # logits scaled by d_kv^-1/2: y and dx can meet the stated bound ...
    for name in ("y", "dx"):
        assert sc[name][0] <= STATED_BF16[0] and sc[name][1] <= STATED_BF16[1], (name, sc[name])
    # ... the weight gradients cannot: every one of them has a mean floor above 2e-3 (each passes at least three
    # bf16 roundings of size 2^-9/sqrt(3) relative, as operands, and the sum over tokens does not average them
    # away relative to the gradient's own size), and the q/k/v gradients a maximum above 2e-2
    for name in grads:
        assert sc[name][1] > STATED_BF16[1], (name, sc[name])
    assert max(sc[n][0] for n in ("wq", "wk", "wv")) > STATED_BF16[0]
    assert max(sc[n][1] for n in grads) < 3.0 * STATED_BF16[1]
    # attn_scale = 1 with unit-variance q, k (logit std 8): every tensor's floor is above the stated bound
    for name in lit:
        assert lit[name][1] > STATED_BF16[1], (name, lit[name])
    assert lit["y"][0] > 3 * STATED_BF16[0] and lit["dx"][1] > 5 * STATED_BF16[1]
    # keeping q and k at ~16 mantissa bits inside the score product does not bring y back under the bound: the
    # rounding of n1 ahead of the q and k projections weighs as much
    sq = floors["literal/split_qk"]
    assert sq["y"][1] > 1.5 * STATED_BF16[1] and sq["y"][0] > 1.5 * STATED_BF16[0]
    # with n1 split as well y lands on the edge of the bound while dx and the gradients stay above it
    sqn = floors["literal/split_qk_n1"]
    assert sqn["y"][1] < 1.1 * STATED_BF16[1]
    assert sqn["dx"][1] > 2.0 * STATED_BF16[1] and sqn["wq"][1] > 2.0 * STATED_BF16[1]


def test_tol_from_floor_rule():
    big = 1 << 30
    assert tol_from_floor((0.9e-2, 1.9e-3), big) == STATED_BF16
    assert tol_from_floor((1.0e-2, 1.99e-3), big) == STATED_BF16
    # a small tensor with the same floor is not held to the stated mean: its mean is itself noisy
    assert tol_from_floor((0.5e-2, 1.93e-3), 128)[1] > 1.4 * 1.93e-3
    t = tol_from_floor((3.0e-2, 1.0e-3), big)
    assert abs(t[0] - max_margin(big) * 3.0e-2) < 1e-12 and t[1] == STATED_BF16[1]
    t = tol_from_floor((0.5e-2, 4.0e-3), big)
    assert t[0] == STATED_BF16[0] and abs(t[1] - MARGIN * 4.0e-3) <= 1e-3 * t[1]
    assert MARGIN <= 1.25 and max_margin(1) == 2.5 and max_margin(99999) == 2.5 and max_margin(100000) == 2.0 and max_margin(big) == 2.0
    # small tensors: the mean of 64 values is itself noisy
    assert abs(mean_margin(64) - (MARGIN + 0.4)) < 1e-12 and mean_margin(10 ** 6) < MARGIN + 0.004
    # ReLU gradients: wider margins for both statistics
    t = tol_from_floor((0.5, 1.0e-2), big, relu=True)
    assert t[0] == 2.5 * 0.5 and abs(t[1] - 1.5e-2) < 1e-5
    assert tol_from_floor((0.5, 1.0e-2), 768, relu=True)[0] == 3.0 * 0.5


def test_spread_between_two_samples_of_the_rounding_noise(monkeypatch):
    """The margins compare two samples of one noise distribution.  The device differs from the model by
    float32-level perturbations of the values that are rounded; here the model is run six times on one case
    with every value perturbed by 3e-7 (relative, Gaussian) before it is rounded.  Only roundings that sit
    on a tie flip at first, but the flips spread down the chain: the six floors of a tensor agree closely in
    the mean of a large tensor, scatter in the mean of a small one, and scatter by tens of percent in the
    maximum -- more than a flat 1.25 allows, within the margins of parity_util."""
    cfg = SI.BlockConfig("floor_spread", 91, batch=2, seq=256, d_model=128, n_heads=2, d_kv=64, d_ff=256,
                         attn_scale=0.125)
    w, x, dy = _case(cfg)
    y, saved = O.block_fwd(cfg, x, w)
    dx, g = O.block_bwd(cfg, dy, w, saved)
    plain = M.rb
    floors = []
    for seed in range(6):
        rng = np.random.default_rng(1000 + seed)
        if seed > 0:
            monkeypatch.setattr(M, "rb", lambda a, rng=rng: plain(np.asarray(a) * (1.0 + 3e-7 * rng.standard_normal(np.shape(a)))))
        floors.append(M.block_floor(cfg, x, w, dy, ref=(y, dx, g)))
    monkeypatch.setattr(M, "rb", plain)
    sizes = {"y": x.size, "dx": x.size, **{k: w[k].size for k in w}}
    worst_max, worst_mean_big = 1.0, 1.0
    for name in floors[0]:
        mx = np.array([f[name][0] for f in floors])
        mn = np.array([f[name][1] for f in floors])
        n = sizes[name]
        assert mx.max() / mx.min() <= max_margin(n), (name, n, mx)
        assert mn.max() / mn.min() <= 1.0 + 3.2 / n ** 0.5 + 0.02, (name, n, mn)
        worst_max = max(worst_max, mx.max() / mx.min())
        if n >= 16384:
            worst_mean_big = max(worst_mean_big, mn.max() / mn.min())
    assert worst_max > 1.25          # a flat 1.25 on the maximum would reject a correct result
    assert worst_mean_big < 1.03     # while the mean of a large tensor is stable
