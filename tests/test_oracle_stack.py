"""Pins for the oracle's stack (embedding, N blocks with a shared bias table, final norm, logits,
cross-entropy with z-loss), CPU only.  Library routines (torch cross_entropy / logsumexp / autograd),
closed forms, invariants and finite differences."""
from dataclasses import replace
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as SI
from oracle import t5_oracle as O
from test_oracle_block import _torch_block

BLK = SI.BlockConfig("stack_tiny", 16, batch=2, seq=10, d_model=16, n_heads=2, d_kv=4, d_ff=24, dtype="f32", causal=True)
TINY = SI.StackConfig("stack_tiny", BLK, n_layers=3, vocab=29, z_loss=1e-2)
TINY_TIED = replace(TINY, name="stack_tiny_tied", tied_logits=True, block=replace(BLK, index=17, causal=False))


def _case(sc):
    w = SI.make_stack_weights(sc)
    SI.make_stack_random_scales(sc, w)
    tokens, targets = SI.make_tokens(sc, ignore_fraction=0.2)
    return w, tokens, targets


# ---------------------------------------------------------------- loss alone
def test_xent_matches_library_cross_entropy_and_logsumexp():
    rng = np.random.default_rng(0)
    logits = rng.standard_normal((4, 7, 33)) * 3
    targets = rng.integers(0, 33, size=(4, 7))
    targets[0, :3] = -1
    loss, lse, n = O.xent_zloss(logits, targets, 0.0)
    ref = F.cross_entropy(torch.from_numpy(logits).reshape(-1, 33), torch.from_numpy(targets).reshape(-1),
                          ignore_index=-1, reduction="mean")
    assert n == 25
    assert abs(loss - float(ref)) < 1e-13
    np.testing.assert_allclose(lse, torch.logsumexp(torch.from_numpy(logits), -1).numpy(), rtol=1e-14)
    z = 0.37
    loss_z, _, _ = O.xent_zloss(logits, targets, z)
    extra = z * (lse[targets >= 0] ** 2).sum() / n
    assert abs(loss_z - (loss + extra)) < 1e-13


def test_xent_closed_forms():
    V = 50
    flat = np.zeros((3, V))
    t = np.array([4, 0, 49])
    loss, lse, n = O.xent_zloss(flat, t, 0.25)
    assert abs(loss - (math.log(V) + 0.25 * math.log(V) ** 2)) < 1e-13      # uniform prediction
    g = O.xent_zloss_grad(flat, t, lse, 0.25, n)
    # every wrong class gets (1 + 2 z lse) / (V n); rows sum to 2 z lse / n
    np.testing.assert_allclose(g[0, 5], (1 + 0.5 * math.log(V)) / V / 3, rtol=1e-13)
    np.testing.assert_allclose(g.sum(-1), 0.5 * math.log(V) / 3, rtol=1e-12)
    # a huge margin for the right class: loss -> z * logit^2 (lse -> logit), CE part -> 0
    big = np.zeros((1, V)); big[0, 7] = 40.0
    loss, _, _ = O.xent_zloss(big, np.array([7]), 0.0)
    assert 0 <= loss < 1e-15
    # adding a constant c to a row shifts lse by c: CE unchanged, z term becomes z (lse + c)^2
    rng = np.random.default_rng(1)
    lg = rng.standard_normal((2, V)); tt = np.array([3, 9])
    l0, lse0, _ = O.xent_zloss(lg, tt, 0.0)
    l1, lse1, _ = O.xent_zloss(lg + 2.5, tt, 0.0)
    assert abs(l0 - l1) < 1e-13 and np.allclose(lse1, lse0 + 2.5, rtol=0, atol=1e-13)
    # no counted position: loss 0 and zero gradient, no division by zero
    l2, lse2, n2 = O.xent_zloss(lg, np.array([-1, -1]), 0.1)
    assert l2 == 0.0 and n2 == 0 and np.all(O.xent_zloss_grad(lg, np.array([-1, -1]), lse2, 0.1, n2) == 0)


def test_xent_grad_against_finite_differences_and_ignored_rows():
    rng = np.random.default_rng(2)
    lg = rng.standard_normal((5, 11)) * 2
    t = np.array([0, 10, -1, 3, 3])
    _, lse, n = O.xent_zloss(lg, t, 0.05)
    g = O.xent_zloss_grad(lg, t, lse, 0.05, n)
    assert np.all(g[2] == 0)
    for (i, j) in [(0, 0), (0, 4), (1, 10), (3, 3), (4, 7), (2, 5)]:
        a, b = lg.copy(), lg.copy()
        a[i, j] += 1e-6; b[i, j] -= 1e-6
        fd = (O.xent_zloss(a, t, 0.05)[0] - O.xent_zloss(b, t, 0.05)[0]) / 2e-6
        assert abs(fd - g[i, j]) < 1e-9


# ---------------------------------------------------------------- whole stack
def _torch_stack_loss(sc, tokens, targets, tw):
    cfg = sc.block
    x = tw["embedding"][torch.from_numpy(tokens).long()]
    for lw in tw["layers"]:
        x = _torch_block(cfg, x, dict(lw, rel_table=tw["rel_table"]))
    nf = F.rms_norm(x, (cfg.d_model,), tw["final_scale"], eps=cfg.rms_eps)
    logits = (nf * cfg.d_model ** -0.5) @ tw["embedding"].T if sc.tied_logits else nf @ tw["logits_w"]
    tt = torch.from_numpy(targets).long()
    lse = torch.logsumexp(logits, -1)
    ce = F.cross_entropy(logits.reshape(-1, sc.vocab), tt.reshape(-1), ignore_index=-1, reduction="sum")
    valid = tt >= 0
    return (ce + sc.z_loss * (lse[valid] ** 2).sum()) / valid.sum()


def _to_torch(w):
    if isinstance(w, dict):
        return {k: _to_torch(v) for k, v in w.items()}
    if isinstance(w, list):
        return [_to_torch(v) for v in w]
    return torch.from_numpy(np.ascontiguousarray(w)).requires_grad_()


@pytest.mark.parametrize("sc", [TINY, TINY_TIED, replace(TINY, n_layers=1, z_loss=0.0)])
def test_stack_loss_and_gradients_against_torch_autograd(sc):
    w, tokens, targets = _case(sc)
    loss, saved = O.stack_loss(sc, tokens, targets, w)
    g = O.stack_loss_grad(sc, w, saved)
    tw = _to_torch(w)
    tl = _torch_stack_loss(sc, tokens, targets, tw)
    tl.backward()
    assert abs(loss - float(tl.detach())) < 1e-12 * max(1.0, abs(loss))
    scale = lambda a: np.sqrt(np.mean(a * a)) + 1e-300
    names = ["embedding", "rel_table", "final_scale"] + ([] if sc.tied_logits else ["logits_w"])
    assert set(g) == set(names) | {"layers"}
    for name in names:
        ref = tw[name].grad.numpy()
        assert np.abs(g[name] - ref).max() / scale(ref) < 1e-9, name
    for l in range(sc.n_layers):
        assert set(g["layers"][l]) == set(w["layers"][l])
        for name, val in g["layers"][l].items():
            ref = tw["layers"][l][name].grad.numpy()
            assert np.abs(val - ref).max() / scale(ref) < 1e-9, (l, name)


def test_shared_table_gradient_is_the_sum_over_layers():
    """Give every layer its own copy of the table: the shared-table gradient is the sum of theirs."""
    sc = TINY
    w, tokens, targets = _case(sc)
    _, saved = O.stack_loss(sc, tokens, targets, w)
    g = O.stack_loss_grad(sc, w, saved)
    tw = _to_torch(w)
    tables = [tw["rel_table"].detach().clone().requires_grad_() for _ in range(sc.n_layers)]
    cfg = sc.block
    x = tw["embedding"][torch.from_numpy(tokens).long()]
    for lw, tab in zip(tw["layers"], tables):
        x = _torch_block(cfg, x, dict(lw, rel_table=tab))
    nf = F.rms_norm(x, (cfg.d_model,), tw["final_scale"], eps=cfg.rms_eps)
    logits = nf @ tw["logits_w"]
    tt = torch.from_numpy(targets).long()
    valid = tt >= 0
    lse = torch.logsumexp(logits, -1)
    loss = (F.cross_entropy(logits.reshape(-1, sc.vocab), tt.reshape(-1), ignore_index=-1, reduction="sum")
            + sc.z_loss * (lse[valid] ** 2).sum()) / valid.sum()
    loss.backward()
    per_layer = [t.grad.numpy() for t in tables]
    assert all(np.abs(p).max() > 0 for p in per_layer)
    np.testing.assert_allclose(g["rel_table"], sum(per_layer), rtol=1e-9, atol=1e-14)


def test_embedding_gradient_rows():
    """Untied: a token that never occurs gets a zero row; a token occurring k times gets the sum of k rows."""
    sc = TINY
    w, tokens, targets = _case(sc)
    tokens = tokens.copy()
    tokens[tokens == 5] = 6                      # token 5 never occurs
    tokens[0, :4] = 11                           # token 11 occurs several times
    _, saved = O.stack_loss(sc, tokens, targets, w)
    g = O.stack_loss_grad(sc, w, saved)
    assert np.all(g["embedding"][5] == 0)
    assert np.abs(g["embedding"][11]).max() > 0
    # moving the whole embedding row of token 11 along a direction changes the loss by <grad row, dir>
    d = np.random.default_rng(4).standard_normal(sc.block.d_model)
    wp = dict(w, embedding=w["embedding"].copy()); wm = dict(w, embedding=w["embedding"].copy())
    wp["embedding"][11] += 1e-6 * d; wm["embedding"][11] -= 1e-6 * d
    fd = (O.stack_loss(sc, tokens, targets, wp)[0] - O.stack_loss(sc, tokens, targets, wm)[0]) / 2e-6
    assert abs(fd - g["embedding"][11] @ d) < 1e-8


def test_zero_output_projections_give_embedding_classifier():
    """With every Wo and Wo_ff at zero the blocks are identities: logits = RMSNorm(E[tokens]) Wout."""
    sc = TINY
    w, tokens, targets = _case(sc)
    for lw in w["layers"]:
        lw["wo"] = np.zeros_like(lw["wo"]); lw["wo_ff"] = np.zeros_like(lw["wo_ff"])
    loss, saved = O.stack_loss(sc, tokens, targets, w)
    x0 = w["embedding"][tokens]
    nf = x0 / np.sqrt((x0 * x0).mean(-1, keepdims=True) + sc.block.rms_eps) * w["final_scale"]
    np.testing.assert_allclose(saved["logits"], nf @ w["logits_w"], rtol=1e-12, atol=1e-13)
    g = O.stack_loss_grad(sc, w, saved)
    assert np.all(g["rel_table"] == 0)           # attention output never reaches the loss


@pytest.mark.parametrize("sc", [TINY, TINY_TIED])
def test_stack_gradients_against_central_differences(sc):
    w, tokens, targets = _case(sc)
    _, saved = O.stack_loss(sc, tokens, targets, w)
    g = O.stack_loss_grad(sc, w, saved)
    rng = np.random.default_rng(9)
    eps = 1e-6

    def probe(get, grad, n_probe=6):
        arr = get(w)
        for fi in rng.choice(arr.size, size=min(n_probe, arr.size), replace=False):
            idx = np.unravel_index(fi, arr.shape)
            old = arr[idx]
            arr[idx] = old + eps; lp = O.stack_loss(sc, tokens, targets, w)[0]
            arr[idx] = old - eps; lm = O.stack_loss(sc, tokens, targets, w)[0]
            arr[idx] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad[idx]) <= 5e-8 * max(1.0, abs(grad[idx]) * 1e2), (idx, fd, grad[idx])

    used = np.unique(tokens)
    probe(lambda ww: ww["rel_table"], g["rel_table"], 12)
    probe(lambda ww: ww["final_scale"], g["final_scale"])
    if not sc.tied_logits:
        probe(lambda ww: ww["logits_w"], g["logits_w"])
    for r, tok in enumerate(used[:3]):
        probe(lambda ww, tok=tok: ww["embedding"][tok], g["embedding"][tok], 3)
    for l in (0, sc.n_layers - 1):
        for name in ("wq", "wo", "wi1", "ln2_scale"):
            probe(lambda ww, l=l, name=name: ww["layers"][l][name], g["layers"][l][name], 3)


# ---------------------------------------------------------------- encoder-decoder model
EC = SI._encdec("ec_tiny", 18, 2, 9, 7, 16, 2, 4, 24, 2, 2, 31, z_loss=1e-2, block=dict(dtype="f32"))
EC_TIED = replace(SI._encdec("ec_tiny_tied", 20, 2, 5, 8, 16, 2, 4, 24, 1, 2, 31, z_loss=0.0, block=dict(dtype="f32")),
                  tied_logits=True)


def _ec_case(ec):
    w = SI.make_encdec_weights(ec)
    SI.make_encdec_random_scales(ec, w)
    return (w,) + SI.make_encdec_tokens(ec, ignore_fraction=0.2)


def _torch_encdec_loss(ec, enc_tokens, dec_tokens, targets, tw):
    from test_oracle_decoder import _torch_decoder_block
    e, d = ec.enc_block, ec.dec_block
    x = tw["embedding"][torch.from_numpy(enc_tokens).long()]
    for lw in tw["enc_layers"]:
        x = _torch_block(e, x, dict(lw, rel_table=tw["enc_rel_table"]))
    enc_out = F.rms_norm(x, (e.d_model,), tw["enc_final_scale"], eps=e.rms_eps)
    x = tw["embedding"][torch.from_numpy(dec_tokens).long()]
    for lw in tw["dec_layers"]:
        x = _torch_decoder_block(d, x, enc_out, dict(lw, rel_table=tw["dec_rel_table"]))
    nf = F.rms_norm(x, (d.d_model,), tw["dec_final_scale"], eps=d.rms_eps)
    logits = (nf * d.d_model ** -0.5) @ tw["embedding"].T if ec.tied_logits else nf @ tw["logits_w"]
    tt = torch.from_numpy(targets).long()
    valid = tt >= 0
    lse = torch.logsumexp(logits, -1)
    ce = F.cross_entropy(logits.reshape(-1, ec.vocab), tt.reshape(-1), ignore_index=-1, reduction="sum")
    return (ce + ec.z_loss * (lse[valid] ** 2).sum()) / valid.sum()


@pytest.mark.parametrize("ec", [EC, EC_TIED])
def test_encdec_loss_and_gradients_against_torch_autograd(ec):
    w, enc_tokens, dec_tokens, targets = _ec_case(ec)
    loss, saved = O.encdec_loss(ec, enc_tokens, dec_tokens, targets, w)
    g = O.encdec_loss_grad(ec, w, saved)
    tw = _to_torch(w)
    tl = _torch_encdec_loss(ec, enc_tokens, dec_tokens, targets, tw)
    tl.backward()
    assert abs(loss - float(tl.detach())) < 1e-12 * max(1.0, abs(loss))
    scale = lambda a: np.sqrt(np.mean(a * a)) + 1e-300
    flat_names = [k for k in w if not k.endswith("_layers")]
    assert set(g) == set(w)
    for name in flat_names:
        ref = tw[name].grad.numpy()
        assert np.abs(g[name] - ref).max() / scale(ref) < 1e-9, name
    for side in ("enc_layers", "dec_layers"):
        for l, lw in enumerate(w[side]):
            assert set(g[side][l]) == set(lw)
            for name, val in g[side][l].items():
                ref = tw[side][l][name].grad.numpy()
                assert np.abs(val - ref).max() / scale(ref) < 1e-9, (side, l, name)


def test_encdec_structure():
    """The decoder sees the encoder only through cross-attention: with every cross-attention output
    projection at zero the loss is that of the decoder stack alone and no gradient reaches the encoder;
    the encoder tokens do not enter the loss as targets, only through enc_out."""
    ec = EC
    w, enc_tokens, dec_tokens, targets = _ec_case(ec)
    for lw in w["dec_layers"]:
        lw["xo"] = np.zeros_like(lw["xo"])
    loss, saved = O.encdec_loss(ec, enc_tokens, dec_tokens, targets, w)
    g = O.encdec_loss_grad(ec, w, saved)
    assert np.all(g["enc_rel_table"] == 0) and np.all(g["enc_final_scale"] == 0)
    assert all(np.all(v == 0) for gl in g["enc_layers"] for v in gl.values())
    sc = SI.StackConfig("dec_only", replace(ec.dec_block, enc_seq=0), ec.n_dec_layers, ec.vocab, z_loss=ec.z_loss)
    strip = lambda lw: {k: v for k, v in lw.items() if k not in ("lnx_scale", "xq", "xk", "xv", "xo")}
    ws = {"embedding": w["embedding"], "rel_table": w["dec_rel_table"], "final_scale": w["dec_final_scale"],
          "logits_w": w["logits_w"], "layers": [strip(lw) for lw in w["dec_layers"]]}
    loss_dec, _ = O.stack_loss(sc, dec_tokens, targets, ws)
    assert abs(loss - loss_dec) < 1e-12
    # other encoder tokens, same loss
    loss2, _ = O.encdec_loss(ec, (enc_tokens + 3) % ec.vocab, dec_tokens, targets, w)
    assert abs(loss2 - loss) < 1e-12


def test_encdec_gradients_against_central_differences():
    ec = EC
    w, enc_tokens, dec_tokens, targets = _ec_case(ec)
    _, saved = O.encdec_loss(ec, enc_tokens, dec_tokens, targets, w)
    g = O.encdec_loss_grad(ec, w, saved)
    rng = np.random.default_rng(10)
    eps = 1e-6

    def probe(arr, grad, n_probe=4):
        for fi in rng.choice(arr.size, size=min(n_probe, arr.size), replace=False):
            idx = np.unravel_index(fi, arr.shape)
            old = arr[idx]
            arr[idx] = old + eps; lp = O.encdec_loss(ec, enc_tokens, dec_tokens, targets, w)[0]
            arr[idx] = old - eps; lm = O.encdec_loss(ec, enc_tokens, dec_tokens, targets, w)[0]
            arr[idx] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad[idx]) <= 5e-8 * max(1.0, abs(grad[idx]) * 1e2), (idx, fd, grad[idx])

    for name in ("enc_rel_table", "dec_rel_table", "enc_final_scale", "dec_final_scale", "logits_w"):
        probe(w[name], g[name], 6)
    both = np.intersect1d(enc_tokens, dec_tokens)
    for tok in list(both[:2]) + [int(enc_tokens[0, 0]), int(dec_tokens[0, 0])]:
        probe(w["embedding"][tok], g["embedding"][tok], 3)
    probe(w["enc_layers"][0]["wk"], g["enc_layers"][0]["wk"])
    probe(w["enc_layers"][1]["wo_ff"], g["enc_layers"][1]["wo_ff"])
    for name in ("xq", "xk", "xv", "xo", "lnx_scale", "wq", "wi0"):
        probe(w["dec_layers"][0][name], g["dec_layers"][0][name], 3)
        probe(w["dec_layers"][1][name], g["dec_layers"][1][name], 3)
