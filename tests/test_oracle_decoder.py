"""Pins for the oracle's decoder block (self-attention, cross-attention, MLP), CPU only.

The cross-attention sublayer is tied to a library routine (torch's scaled_dot_product_attention
with rectangular shapes), to invariants of attention without positions (the encoder tokens form a
set), to a closed form (one encoder token), to torch autograd and to finite differences.
"""
from dataclasses import replace

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as SI
from oracle import t5_oracle as O
from test_oracle_block import _torch_block

DEC = SI.BlockConfig("dec_tiny", 12, batch=2, seq=10, d_model=16, n_heads=2, d_kv=4, d_ff=24, dtype="f32",
                     causal=True, enc_seq=7)
DEC_LONG_ENC = replace(DEC, name="dec_tiny_long_enc", index=13, seq=6, enc_seq=19, attn_scale=0.5)


def _case(cfg):
    w = SI.make_weights(cfg)
    w.update(SI.make_random_scales(cfg))
    x, dy = SI.make_activations(cfg)
    enc = SI.make_encoder_output(cfg)
    return w, x, enc, dy


def test_input_generator_shapes():
    w, x, enc, dy = _case(DEC)
    assert enc.shape == (DEC.batch, DEC.enc_seq, DEC.d_model)
    for name in ("xq", "xk", "xv"):
        assert w[name].shape == (DEC.d_model, DEC.inner)
    assert w["xo"].shape == (DEC.inner, DEC.d_model)
    assert w["lnx_scale"].shape == (DEC.d_model,)
    # the encoder-block tensors of a config do not move when cross-attention is added
    w0 = SI.make_weights(replace(DEC, enc_seq=0))
    for name in w0:
        np.testing.assert_array_equal(w0[name], SI.make_weights(DEC)[name])


@pytest.mark.parametrize("cfg", [DEC, DEC_LONG_ENC])
def test_cross_attention_matches_library_rectangular_attention(cfg):
    cfg = replace(cfg, attn_scale=cfg.d_kv ** -0.5)
    w, x, enc, _ = _case(cfg)
    _, sv = O.decoder_block_fwd(cfg, x, enc, w)
    assert sv["px"].shape == (cfg.batch, cfg.n_heads, cfg.seq, cfg.enc_seq)
    np.testing.assert_allclose(sv["px"].sum(-1), 1.0, rtol=0, atol=1e-14)
    ref = F.scaled_dot_product_attention(*(torch.from_numpy(sv[n]) for n in ("qx", "kx", "vx")))
    ref = ref.permute(0, 2, 1, 3).reshape(cfg.batch, cfg.seq, cfg.inner).numpy()
    np.testing.assert_allclose(sv["cx"], ref, rtol=1e-12, atol=1e-13)
    # keys and values come from the encoder output, queries from the decoder stream
    np.testing.assert_allclose(sv["kx"][1, 1, 3], (enc[1, 3] @ w["xk"])[cfg.d_kv:2 * cfg.d_kv], rtol=1e-13)
    np.testing.assert_allclose(sv["vx"][0, 0, 2], (enc[0, 2] @ w["xv"])[:cfg.d_kv], rtol=1e-13)
    np.testing.assert_allclose(sv["qx"][1, 0, 4], (sv["nx"][1, 4] @ w["xq"])[:cfg.d_kv], rtol=1e-13)


def test_self_attention_sublayer_is_the_plain_block():
    """With the cross-attention output projection at zero the decoder block is the causal block."""
    w, x, enc, dy = _case(DEC)
    w["xo"] = np.zeros_like(w["xo"])
    y, sv = O.decoder_block_fwd(DEC, x, enc, w)
    y0, _ = O.block_fwd(DEC, x, {k: w[k] for k in w if k[0] != "x" and k != "lnx_scale"})
    np.testing.assert_allclose(y, y0, rtol=1e-13, atol=1e-14)
    _, denc, g = O.decoder_block_bwd(DEC, dy, w, sv)
    assert np.all(denc == 0) and np.all(g["xq"] == 0) and np.all(g["xk"] == 0) and np.all(g["xv"] == 0)
    assert np.any(g["xo"] != 0)


def test_encoder_tokens_form_a_set():
    """No bias, no mask: permuting the encoder tokens leaves y unchanged and permutes denc."""
    w, x, enc, dy = _case(DEC)
    y, sv = O.decoder_block_fwd(DEC, x, enc, w)
    dx, denc, g = O.decoder_block_bwd(DEC, dy, w, sv)
    perm = np.random.default_rng(5).permutation(DEC.enc_seq)
    y2, sv2 = O.decoder_block_fwd(DEC, x, enc[:, perm], w)
    dx2, denc2, g2 = O.decoder_block_bwd(DEC, dy, w, sv2)
    np.testing.assert_allclose(y2, y, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dx2, dx, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(denc2, denc[:, perm], rtol=1e-11, atol=1e-12)
    for name in g:
        np.testing.assert_allclose(g2[name], g[name], rtol=1e-10, atol=1e-11, err_msg=name)


def test_decoder_tokens_do_not_mix_in_cross_attention():
    """Cross-attention is per query: with the self-attention output off, y[b, i] depends on x[b, i] only."""
    w, x, enc, _ = _case(DEC)
    w["wo"] = np.zeros_like(w["wo"])
    y, _ = O.decoder_block_fwd(DEC, x, enc, w)
    x2 = x.copy()
    x2[:, 3] += 1.0
    y2, _ = O.decoder_block_fwd(DEC, x2, enc, w)
    changed = np.abs(y2 - y).max(axis=(0, 2)) > 0
    assert changed.tolist() == [i == 3 for i in range(DEC.seq)]


def test_single_encoder_token_closed_form():
    """S_enc = 1: softmax over one key is 1, so cx = enc Xv for every query and
    h2 = h1 + enc Xv Xo; no gradient reaches Xq, Xk or the cross-attention norm scale."""
    cfg = replace(DEC, enc_seq=1)
    w, x, enc, dy = _case(cfg)
    y, sv = O.decoder_block_fwd(cfg, x, enc, w)
    np.testing.assert_allclose(sv["h2"], sv["h1"] + (enc @ w["xv"] @ w["xo"]), rtol=1e-13, atol=1e-14)
    _, denc, g = O.decoder_block_bwd(cfg, dy, w, sv)
    for name in ("xq", "xk", "lnx_scale"):
        assert np.abs(g[name]).max() < 1e-15, name
    # dh2 (rebuilt here from the MLP sublayer) summed over queries flows back through Xo^T then Xv^T
    da = dy @ w["wo_ff"].T
    du = da * sv["wl"] * O.gelu_grad(sv["u"])
    dwl = da * O.gelu(sv["u"])
    dh2 = dy + O.rmsnorm_bwd(sv["h2"], w["ln2_scale"], sv["r2"], du @ w["wi0"].T + dwl @ w["wi1"].T)[0]
    np.testing.assert_allclose(denc[:, 0], dh2.sum(1) @ w["xo"].T @ w["xv"].T, rtol=1e-11, atol=1e-12)


def _torch_decoder_block(cfg, x, enc, w):
    """Independent forward from torch library ops; the self-attention + MLP part is the block's."""
    B, S, H, K = cfg.batch, cfg.seq, cfg.n_heads, cfg.d_kv
    n1 = F.rms_norm(x, (cfg.d_model,), w["ln1_scale"], eps=cfg.rms_eps)
    from test_oracle_block import _bucket_from_fixture
    idx = torch.tensor([[_bucket_from_fixture(j - i, cfg.causal) for j in range(S)] for i in range(S)])
    heads = lambda t, m: torch.einsum("bsd,dhk->bhsk", t, m.view(cfg.d_model, H, K))
    q, k, v = heads(n1, w["wq"]), heads(n1, w["wk"]), heads(n1, w["wv"])
    logits = cfg.attn_scale * torch.einsum("bhik,bhjk->bhij", q, k) + w["rel_table"][idx].permute(2, 0, 1)
    if cfg.causal:
        logits = logits.masked_fill(~torch.ones(S, S, dtype=torch.bool).tril(), float("-inf"))
    o = torch.einsum("bhij,bhjk->bihk", F.softmax(logits, dim=-1), v).reshape(B, S, H * K)
    h1 = x + o @ w["wo"]
    nx = F.rms_norm(h1, (cfg.d_model,), w["lnx_scale"], eps=cfg.rms_eps)
    ox = F.scaled_dot_product_attention(heads(nx, w["xq"]), heads(enc, w["xk"]), heads(enc, w["xv"]),
                                        scale=cfg.attn_scale)
    h2 = h1 + ox.permute(0, 2, 1, 3).reshape(B, S, H * K) @ w["xo"]
    n2 = F.rms_norm(h2, (cfg.d_model,), w["ln2_scale"], eps=cfg.rms_eps)
    from test_oracle_block import _torch_mlp
    return h2 + _torch_mlp(cfg, n2, w)


@pytest.mark.parametrize("cfg", [DEC, DEC_LONG_ENC, replace(DEC, causal=False, index=14),
                                 replace(DEC, mlp="relu", index=16), replace(DEC, mlp="geglu_erf", index=17),
                                 replace(SI.CONFIGS["c1_tiny_f32"], causal=True, enc_seq=96, batch=1, index=15)])
def test_forward_and_backward_against_torch_autograd(cfg):
    w, x, enc, dy = _case(cfg)
    y, sv = O.decoder_block_fwd(cfg, x, enc, w)
    dx, denc, g = O.decoder_block_bwd(cfg, dy, w, sv)
    tw = {k_: torch.from_numpy(np.ascontiguousarray(v)).requires_grad_() for k_, v in w.items()}
    tx = torch.from_numpy(x).requires_grad_()
    te = torch.from_numpy(enc).requires_grad_()
    ty = _torch_decoder_block(cfg, tx, te, tw)
    ty.backward(torch.from_numpy(dy))
    np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-11, atol=1e-12)
    scale = lambda a: np.sqrt(np.mean(a * a)) + 1e-300
    assert np.abs(dx - tx.grad.numpy()).max() / scale(dx) < 1e-10
    assert np.abs(denc - te.grad.numpy()).max() / scale(denc) < 1e-10
    assert set(g) == set(w)
    for name, val in g.items():
        ref = tw[name].grad.numpy()
        assert val.shape == ref.shape
        assert np.abs(val - ref).max() / scale(ref) < 1e-10, name


@pytest.mark.parametrize("cfg", [DEC, DEC_LONG_ENC])
def test_backward_against_central_differences(cfg):
    w, x, enc, dy = _case(cfg)
    y, sv = O.decoder_block_fwd(cfg, x, enc, w)
    dx, denc, g = O.decoder_block_bwd(cfg, dy, w, sv)
    loss = lambda xx, ee, ww: float(np.sum(O.decoder_block_fwd(cfg, xx, ee, ww)[0] * dy))
    rng = np.random.default_rng(23)
    eps = 1e-6

    def check(name, arr, grad, n_probe=10):
        for fi in rng.choice(arr.size, size=min(n_probe, arr.size), replace=False):
            idx = np.unravel_index(fi, arr.shape)
            ap, am = arr.copy(), arr.copy()
            ap[idx] += eps
            am[idx] -= eps
            if name == "x":
                fd = (loss(ap, enc, w) - loss(am, enc, w)) / (2 * eps)
            elif name == "enc":
                fd = (loss(x, ap, w) - loss(x, am, w)) / (2 * eps)
            else:
                wp, wm = dict(w), dict(w)
                wp[name], wm[name] = ap, am
                fd = (loss(x, enc, wp) - loss(x, enc, wm)) / (2 * eps)
            assert abs(fd - grad[idx]) <= 2e-6 * max(1.0, abs(grad[idx])), (name, idx, fd, grad[idx])

    check("x", x, dx)
    check("enc", enc, denc)
    for name in w:
        check(name, w[name], g[name], n_probe=8)
