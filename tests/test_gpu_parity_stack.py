"""GPU parity of the layer stack (embedding, N blocks with a shared bias table, final norm, logits,
cross-entropy with z-loss; forward + backward in one call) through the C ABI against the float64 oracle."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import synth_inputs as SI
from oracle import t5_oracle as O
from parity_util import TOL_F32, check_bf16, general_mlp_path, is_relu, rel_err, to_dev, to_np

pytestmark = pytest.mark.gpu

BLK = SI.BlockConfig("stack_f32", 60, batch=2, seq=24, d_model=32, n_heads=2, d_kv=8, d_ff=48, dtype="f32", causal=True)
F32_CASES = [
    SI.StackConfig("stack_f32", BLK, n_layers=3, vocab=29, z_loss=1e-2),                       # odd vocab: generic loss kernel
    SI.StackConfig("stack_f32_tied", replace(BLK, index=61, causal=False), n_layers=2, vocab=64, tied_logits=True,
                   z_loss=1e-3),                                                               # 16-byte rows: register loss kernel
    SI.StackConfig("stack_f32_remat", replace(BLK, index=62), n_layers=3, vocab=40, remat=True, z_loss=0.0),
    SI.StackConfig("stack_f32_relu", replace(BLK, index=68, mlp="relu"), n_layers=2, vocab=40, z_loss=1e-3),
    SI.StackConfig("stack_f32_wide_vocab", replace(BLK, index=63, batch=1, seq=16), n_layers=1, vocab=5000, z_loss=1e-4),
]


def _case(sc, ignore_fraction=0.15):
    w = SI.make_stack_weights(sc)
    SI.make_stack_random_scales(sc, w)
    tokens, targets = SI.make_tokens(sc, ignore_fraction=ignore_fraction)
    return w, tokens, targets


def _upload(sc, w, tokens, targets):
    dt = sc.block.dtype
    dw = {k: to_dev(v, dt) for k, v in w.items() if k != "layers"}
    dw["layers"] = [{k: to_dev(v, dt) for k, v in lw.items()} for lw in w["layers"]]
    return dw, torch.from_numpy(tokens).cuda(), torch.from_numpy(targets).cuda()


def _run(sc, w, tokens, targets, **kw):
    import paper_2203_17189_amd as P
    dw, tt, tg = _upload(sc, w, tokens, targets)
    loss, grads = P.t5_stack_loss_and_grad(sc, tt, tg, dw, **kw)
    torch.cuda.synchronize()
    return float(loss.item()), grads


def _stack_errs(sc, got, g, tokens, targets):
    """{name: (max, mean)} of a gradient set `got` (numpy, nested like g) against the oracle's g.  The embedding
    gradient (untied) is non-zero only in the rows of tokens that occur and the output-matrix gradient is
    dominated by the columns of targets that occur: their error is scaled by the RMS over that support."""
    errs = {}
    for name in [k for k in g if k != "layers"]:
        rms = None
        if name == "embedding" and not sc.tied_logits:
            rows = np.unique(tokens)
            rms = float(np.sqrt(np.mean(g[name][rows] ** 2)))
        if name == "logits_w":
            cols = np.unique(targets[targets >= 0])
            rms = float(np.sqrt(np.mean(g[name][:, cols] ** 2)))
        errs[name] = rel_err(got[name], g[name], rms)
    for l in range(sc.n_layers):
        for name, val in g["layers"][l].items():
            errs[f"L{l}.{name}"] = rel_err(got["layers"][l][name], val)
    return errs


def _grads_np(gg):
    return {k: ([{n: to_np(t) for n, t in d.items()} for d in v] if k.endswith("layers") else to_np(v)) for k, v in gg.items()}


def _compare(sc, tol_loss, tol=None, verbose=True):
    """tol: a plain bound on the maximum (float32 stacks).  None (bf16 stacks): every tensor is held to the bound
    derived from its floor under ideal bf16-operand arithmetic (tests/bf16_model.stack_model, same case)."""
    w, tokens, targets = _case(sc)
    loss, saved = O.stack_loss(sc, tokens, targets, w)
    g = O.stack_loss_grad(sc, w, saved)
    gl, gg = _run(sc, w, tokens, targets)
    got = _grads_np(gg)
    if not sc.tied_logits:      # rows of tokens that do not occur receive nothing at all
        rows = np.unique(tokens)
        assert np.all(got["embedding"][np.setdiff1d(np.arange(sc.vocab), rows)] == 0)
    errs = _stack_errs(sc, got, g, tokens, targets)
    if verbose:
        worst = sorted(errs.items(), key=lambda kv: -kv[1][0])[:6]
        print(sc.name, "loss", gl, loss, "worst", [(k, tuple(round(x, 5) for x in v)) for k, v in worst])
    assert abs(gl - loss) <= tol_loss * max(1.0, abs(loss)), (gl, loss)
    if tol is not None:
        for k, e in errs.items():
            assert e[0] <= tol, (k, e)
        return errs
    import bf16_model as M
    _, mg = M.stack_model(sc, tokens, targets, w, round_uw=general_mlp_path(sc.block))
    check_bf16(sc.name, errs, _stack_errs(sc, mg, g, tokens, targets), relu=is_relu(sc.block))
    return errs


@pytest.mark.parametrize("sc", F32_CASES, ids=[c.name for c in F32_CASES])
def test_stack_f32(sc):
    _compare(sc, 1e-5, TOL_F32[0])


def test_stack_loss_only_accumulate_and_no_targets():
    import paper_2203_17189_amd as P
    sc = F32_CASES[0]
    w, tokens, targets = _case(sc)
    dw, tt, tg = _upload(sc, w, tokens, targets)
    loss, g1 = P.t5_stack_loss_and_grad(sc, tt, tg, dw)
    loss_only, none = P.t5_stack_loss_and_grad(sc, tt, tg, dw, want_grads=False)
    assert none is None and torch.equal(loss, loss_only)
    clone = lambda g: {k: ([{n: t.clone() for n, t in d.items()} for d in v] if k == "layers" else v.clone())
                       for k, v in g.items()}
    g2 = clone(g1)
    P.t5_stack_loss_and_grad(sc, tt, tg, dw, grads=g2, accumulate=True)
    torch.cuda.synchronize()
    for k in ("embedding", "rel_table", "final_scale", "logits_w"):
        np.testing.assert_allclose(to_np(g2[k]), 2 * to_np(g1[k]), rtol=2e-5, atol=1e-7)
    for l in range(sc.n_layers):
        for n in g1["layers"][l]:
            np.testing.assert_allclose(to_np(g2["layers"][l][n]), 2 * to_np(g1["layers"][l][n]), rtol=2e-5, atol=1e-7)
    # no position carries a loss: zero loss, zero gradients, no division by zero
    none_t = torch.full_like(tg, -1)
    loss0, g0 = P.t5_stack_loss_and_grad(sc, tt, none_t, dw)
    torch.cuda.synchronize()
    assert float(loss0.item()) == 0.0
    assert all(float(g0[k].abs().max()) == 0.0 for k in ("embedding", "rel_table", "final_scale", "logits_w"))
    # out-of-range targets are ignored like negative ones
    big_t = torch.where(tg < 0, torch.full_like(tg, sc.vocab + 5), tg)
    loss_b, _ = P.t5_stack_loss_and_grad(sc, tt, big_t, dw, want_grads=False)
    assert torch.equal(loss_b, loss)


BF_BLK = SI.BlockConfig("stack_bf16", 64, batch=2, seq=128, d_model=128, n_heads=2, d_kv=64, d_ff=256, causal=True,
                        attn_scale=64 ** -0.5)
BF16_CASES = [
    SI.StackConfig("stack_bf16", BF_BLK, n_layers=2, vocab=512),
    SI.StackConfig("stack_bf16_tied", replace(BF_BLK, index=65, causal=False), n_layers=2, vocab=512, tied_logits=True),
    SI.StackConfig("stack_bf16_t5_vocab", replace(BF_BLK, index=66, batch=1, d_model=64, n_heads=1, d_ff=128),
                   n_layers=1, vocab=32128),
    SI.StackConfig("stack_bf16_relu_tied", replace(BF_BLK, index=69, mlp="relu"), n_layers=2, vocab=512, tied_logits=True),
    # more tokens than one logits chunk (16384) and not a multiple of it: two launches of the head, the second short
    SI.StackConfig("stack_bf16_two_chunks", replace(BF_BLK, index=59, batch=130, seq=128, d_model=64, n_heads=1, d_ff=64),
                   n_layers=1, vocab=256),
    SI.StackConfig("stack_bf16_ragged", SI.BlockConfig("stack_bf16_ragged", 67, batch=1, seq=50, d_model=72, n_heads=3,
                                                        d_kv=24, d_ff=136, causal=True, attn_scale=24 ** -0.5),
                   n_layers=2, vocab=301),
]


@pytest.mark.parametrize("sc", BF16_CASES, ids=[c.name for c in BF16_CASES])
def test_stack_bf16_small(sc):
    _compare(sc, 5e-4)


def test_stack_bf16_accumulate_with_grouped_weight_gradients():
    """A second call with accumulate adds to the gradients of the first, also where the weight gradients of
    all layers come from the grouped launches (bf16, activations kept)."""
    import paper_2203_17189_amd as P
    sc = replace(BF16_CASES[0], n_layers=3)
    w, tokens, targets = _case(sc)
    dw, tt, tg = _upload(sc, w, tokens, targets)
    _, g1 = P.t5_stack_loss_and_grad(sc, tt, tg, dw)
    g2 = {k: ([{n: t.clone() for n, t in d.items()} for d in v] if k == "layers" else v.clone()) for k, v in g1.items()}
    P.t5_stack_loss_and_grad(sc, tt, tg, dw, grads=g2, accumulate=True)
    torch.cuda.synchronize()
    close = lambda a, b, what: np.testing.assert_allclose(to_np(a), 2 * to_np(b), rtol=0, atol=1e-4 * float(b.abs().max()) + 1e-12, err_msg=str(what))
    for k in ("embedding", "rel_table", "final_scale", "logits_w"):
        close(g2[k], g1[k], k)
    for l in range(sc.n_layers):
        for n in g1["layers"][l]:
            close(g2["layers"][l][n], g1["layers"][l][n], (l, n))


def test_stack_bf16_remat_matches_stashed():
    """Recomputing each layer inside the backward sweep gives the same loss bit for bit and the same
    gradients up to the order of the float32 atomic additions."""
    sc = BF16_CASES[0]
    w, tokens, targets = _case(sc)
    l1, g1 = _run(sc, w, tokens, targets)
    l2, g2 = _run(replace(sc, remat=True), w, tokens, targets)
    assert l1 == l2
    for k in ("embedding", "rel_table", "final_scale", "logits_w"):
        a = to_np(g1[k]); assert np.abs(to_np(g2[k]) - a).max() <= 1e-4 * np.abs(a).max(), k
    for l in range(sc.n_layers):
        for n in g1["layers"][l]:
            a = to_np(g1["layers"][l][n]); assert np.abs(to_np(g2["layers"][l][n]) - a).max() <= 1e-4 * np.abs(a).max(), (l, n)


def test_stack_named_config_reduced_batch():
    """T5.1.1-Base decoder-only stack at its real depth, widths, length and vocabulary, one sequence."""
    sc = replace(SI.STACK_CONFIGS["s1_lm_base"].with_batch(1), name="s1_lm_base_b1")
    sc = replace(sc, block=replace(sc.block, attn_scale=64 ** -0.5))
    _compare(sc, 5e-4)


# ---------------------------------------------------------------- encoder-decoder model
def _ec_upload(ec, w, enc_tokens, dec_tokens, targets):
    dt = ec.dec_block.dtype
    dw = {k: to_dev(v, dt) for k, v in w.items() if not k.endswith("_layers")}
    for side in ("enc_layers", "dec_layers"):
        dw[side] = [{k: to_dev(v, dt) for k, v in lw.items()} for lw in w[side]]
    dev = lambda a: torch.from_numpy(a).cuda()
    return dw, dev(enc_tokens), dev(dec_tokens), dev(targets)


def _ec_errs(ec, got, g, enc_tokens, dec_tokens, targets):
    errs = {}
    for name in [k for k in g if not k.endswith("_layers")]:
        rms = None
        if name == "embedding" and not ec.tied_logits:
            rows = np.unique(np.concatenate([enc_tokens.ravel(), dec_tokens.ravel()]))
            rms = float(np.sqrt(np.mean(g[name][rows] ** 2)))
        if name == "logits_w":
            cols = np.unique(targets[targets >= 0])
            rms = float(np.sqrt(np.mean(g[name][:, cols] ** 2)))
        errs[name] = rel_err(got[name], g[name], rms)
    for side in ("enc_layers", "dec_layers"):
        for l, gl_ in enumerate(g[side]):
            for name, val in gl_.items():
                errs[f"{side[:3]}{l}.{name}"] = rel_err(got[side][l][name], val)
    return errs


def _ec_compare(ec, tol_loss, tol=None):
    """tol as in _compare: a plain bound (float32), or None for the floor-derived bounds (bf16)."""
    import paper_2203_17189_amd as P
    w = SI.make_encdec_weights(ec)
    SI.make_encdec_random_scales(ec, w)
    enc_tokens, dec_tokens, targets = SI.make_encdec_tokens(ec, ignore_fraction=0.15)
    loss, saved = O.encdec_loss(ec, enc_tokens, dec_tokens, targets, w)
    g = O.encdec_loss_grad(ec, w, saved)
    dw, te, td, tg = _ec_upload(ec, w, enc_tokens, dec_tokens, targets)
    gl, gg = P.t5_encdec_loss_and_grad(ec, te, td, tg, dw)
    torch.cuda.synchronize()
    gl = float(gl.item())
    errs = _ec_errs(ec, _grads_np(gg), g, enc_tokens, dec_tokens, targets)
    worst = sorted(errs.items(), key=lambda kv: -kv[1][0])[:6]
    print(ec.name, "loss", gl, loss, "worst", [(k, tuple(round(x, 5) for x in v)) for k, v in worst])
    assert abs(gl - loss) <= tol_loss * max(1.0, abs(loss)), (gl, loss)
    if tol is not None:
        for k, e in errs.items():
            assert e[0] <= tol, (k, e)
        return
    import bf16_model as M
    _, mg = M.encdec_model(ec, enc_tokens, dec_tokens, targets, w,
                           round_uw=general_mlp_path(ec.enc_block) or general_mlp_path(ec.dec_block))
    check_bf16(ec.name, errs, _ec_errs(ec, mg, g, enc_tokens, dec_tokens, targets),
               relu=is_relu(ec.enc_block) or is_relu(ec.dec_block))


EC_F32 = [
    SI._encdec("ec_f32", 70, 2, 20, 12, 32, 2, 8, 48, 2, 2, 37, z_loss=1e-2, block=dict(dtype="f32")),
    replace(SI._encdec("ec_f32_tied_remat", 72, 1, 9, 17, 32, 2, 8, 48, 1, 3, 64, z_loss=1e-3, block=dict(dtype="f32")),
            tied_logits=True, remat=True),
]


@pytest.mark.parametrize("ec", EC_F32, ids=[c.name for c in EC_F32])
def test_encdec_f32(ec):
    _ec_compare(ec, 1e-5, TOL_F32[0])


EC_BF16 = [
    SI._encdec("ec_bf16", 74, 2, 256, 128, 128, 2, 64, 256, 2, 2, 512, block=dict(attn_scale=64 ** -0.5)),
    replace(SI._encdec("ec_bf16_remat", 76, 1, 128, 128, 128, 2, 64, 256, 1, 2, 512, block=dict(attn_scale=64 ** -0.5)),
            remat=True),
    SI._encdec("ec_bf16_ragged", 78, 1, 70, 33, 72, 3, 24, 136, 2, 1, 301, block=dict(attn_scale=24 ** -0.5)),
]


@pytest.mark.parametrize("ec", EC_BF16, ids=[c.name for c in EC_BF16])
def test_encdec_bf16_small(ec):
    # a gradient in the encoder has crossed every decoder layer and the encoder layers above it
    _ec_compare(ec, 5e-4)


def test_encdec_named_config_reduced_batch():
    """T5.1.1-Base encoder-decoder at its real depth, widths, lengths and vocabulary, one sequence pair."""
    ec = SI.ENCDEC_CONFIGS["e1_t5_base"].with_batch(1)
    ec = replace(ec, enc_block=replace(ec.enc_block, attn_scale=64 ** -0.5),
                 dec_block=replace(ec.dec_block, attn_scale=64 ** -0.5))
    _ec_compare(ec, 5e-4)
