"""Pins for the oracle's dropout beyond the single block (CPU only): the decoder layer's six sites, and
the stacks' per-layer seeds and end sites.  The masks are rebuilt here from the stated recipe (site number,
row and column meaning, layer-seed formula) and handed to torch library ops as constants; torch autograd
then fixes forward and backward."""
from dataclasses import replace

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as SI
from oracle import t5_oracle as O
from test_oracle_block import _bucket_from_fixture, _torch_mlp
from test_oracle_decoder import DEC, DEC_LONG_ENC, _case as _dec_case
from test_oracle_dropout import _torch_block_drop
from test_oracle_stack import EC, EC_TIED, TINY, TINY_TIED, _case as _stack_case, _ec_case, _to_torch

M64 = (1 << 64) - 1
GOLD = 0x9E3779B97F4A7C15


def _mask(seed, site, rows, cols, rate, shape):
    return (O.dropout_keep(seed, site, rows, cols, rate) / (1.0 - rate)).reshape(shape)


def _block_masks(cfg, seed):
    B, S, H, d, f, p = cfg.batch, cfg.seq, cfg.n_heads, cfg.d_model, cfg.d_ff, cfg.dropout_rate
    return {1: _mask(seed, 1, B * H * S, S, p, (B, H, S, S)), 2: _mask(seed, 2, B * S, d, p, (B, S, d)),
            3: _mask(seed, 3, B * S, f, p, (B, S, f)), 4: _mask(seed, 4, B * S, d, p, (B, S, d))}


def _decoder_masks(cfg, seed, enc_seq):
    B, S, H, d, p = cfg.batch, cfg.seq, cfg.n_heads, cfg.d_model, cfg.dropout_rate
    m = _block_masks(cfg, seed)
    m[5] = _mask(seed, 5, B * H * S, enc_seq, p, (B, H, S, enc_seq))
    m[6] = _mask(seed, 6, B * S, d, p, (B, S, d))
    return m


def _torch_decoder_block_drop(cfg, x, enc, w, masks):
    B, S, H, K = cfg.batch, cfg.seq, cfg.n_heads, cfg.d_kv
    m = {k: torch.from_numpy(v) for k, v in masks.items()}
    heads = lambda t, mm: torch.einsum("bsd,dhk->bhsk", t, mm.view(cfg.d_model, H, K))
    n1 = F.rms_norm(x, (cfg.d_model,), w["ln1_scale"], eps=cfg.rms_eps)
    q, k, v = heads(n1, w["wq"]), heads(n1, w["wk"]), heads(n1, w["wv"])
    idx = torch.tensor([[_bucket_from_fixture(j - i, cfg.causal) for j in range(S)] for i in range(S)])
    logits = cfg.attn_scale * torch.einsum("bhik,bhjk->bhij", q, k) + w["rel_table"][idx].permute(2, 0, 1)
    if cfg.causal:
        logits = logits.masked_fill(~torch.ones(S, S, dtype=torch.bool).tril(), float("-inf"))
    o = torch.einsum("bhij,bhjk->bihk", F.softmax(logits, dim=-1) * m[1], v).reshape(B, S, H * K)
    h1 = x + (o @ w["wo"]) * m[2]
    nx = F.rms_norm(h1, (cfg.d_model,), w["lnx_scale"], eps=cfg.rms_eps)
    qx, kx, vx = heads(nx, w["xq"]), heads(enc, w["xk"]), heads(enc, w["xv"])
    px = F.softmax(cfg.attn_scale * torch.einsum("bhik,bhjk->bhij", qx, kx), dim=-1) * m[5]
    ox = torch.einsum("bhij,bhjk->bihk", px, vx).reshape(B, S, H * K)
    h2 = h1 + (ox @ w["xo"]) * m[6]
    n2 = F.rms_norm(h2, (cfg.d_model,), w["ln2_scale"], eps=cfg.rms_eps)
    if cfg.mlp == "relu":
        a = F.relu(n2 @ w["wi0"])
    else:
        a = F.gelu(n2 @ w["wi0"], approximate="tanh") * (n2 @ w["wi1"])
    return h2 + ((a * m[3]) @ w["wo_ff"]) * m[4]


DEC_DROP = replace(DEC, name="dec_tiny_drop", index=32, dropout_rate=0.25, dropout_seed=0xABCDEF0123456789)
DEC_DROP_LONG = replace(DEC_LONG_ENC, name="dec_tiny_drop_long", index=33, dropout_rate=0.1, dropout_seed=3, mlp="relu")


@pytest.mark.parametrize("cfg", [DEC_DROP, DEC_DROP_LONG])
def test_decoder_block_with_dropout_against_torch_autograd(cfg):
    w, x, enc, dy = _dec_case(cfg)
    y, sv = O.decoder_block_fwd(cfg, x, enc, w)
    dx, denc, g = O.decoder_block_bwd(cfg, dy, w, sv)
    tw = {k_: torch.from_numpy(np.ascontiguousarray(v)).requires_grad_() for k_, v in w.items()}
    tx, te = torch.from_numpy(x).requires_grad_(), torch.from_numpy(enc).requires_grad_()
    ty = _torch_decoder_block_drop(cfg, tx, te, tw, _decoder_masks(cfg, cfg.dropout_seed, cfg.enc_seq))
    ty.backward(torch.from_numpy(dy))
    np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-11, atol=1e-12)
    scale = lambda a: np.sqrt(np.mean(a * a)) + 1e-300
    assert np.abs(dx - tx.grad.numpy()).max() / scale(dx) < 1e-10
    assert np.abs(denc - te.grad.numpy()).max() / scale(denc) < 1e-10
    for name, val in g.items():
        assert np.abs(val - tw[name].grad.numpy()).max() / scale(val) < 1e-10, name
    # rate 0 is the plain layer, bit for bit
    y0, _ = O.decoder_block_fwd(replace(cfg, dropout_rate=0.0), x, enc, w)
    y1, _ = O.decoder_block_fwd(replace(cfg, dropout_rate=0.0, dropout_seed=1), x, enc, w)
    assert np.array_equal(y0, y1) and np.abs(y0 - y).max() > 1e-3


def test_layer_seed_formula():
    assert O.dropout_layer_seed(0, 0) == GOLD
    assert O.dropout_layer_seed(M64, 0) == GOLD - 1                      # wraps mod 2^64
    assert O.dropout_layer_seed(5, 2) == (5 + 3 * GOLD) & M64
    assert len({O.dropout_layer_seed(7, l) for l in range(64)}) == 64


def _torch_stack_loss_drop(sc, tokens, targets, tw):
    cfg = sc.block
    B, S, d, p, seed = cfg.batch, cfg.seq, cfg.d_model, cfg.dropout_rate, cfg.dropout_seed
    x = tw["embedding"][torch.from_numpy(tokens).long()] * torch.from_numpy(_mask(seed, 7, B * S, d, p, (B, S, d)))
    for l, lw in enumerate(tw["layers"]):
        x = _torch_block_drop(cfg, x, dict(lw, rel_table=tw["rel_table"]), _block_masks(cfg, (seed + (l + 1) * GOLD) & M64))
    nf = F.rms_norm(x, (d,), tw["final_scale"], eps=cfg.rms_eps) * torch.from_numpy(_mask(seed, 8, B * S, d, p, (B, S, d)))
    logits = (nf * d ** -0.5) @ tw["embedding"].T if sc.tied_logits else nf @ tw["logits_w"]
    tt = torch.from_numpy(targets).long()
    lse = torch.logsumexp(logits, -1)
    ce = F.cross_entropy(logits.reshape(-1, sc.vocab), tt.reshape(-1), ignore_index=-1, reduction="sum")
    valid = tt >= 0
    return (ce + sc.z_loss * (lse[valid] ** 2).sum()) / valid.sum()


def _drop_stack(sc, rate, seed):
    return replace(sc, block=replace(sc.block, dropout_rate=rate, dropout_seed=seed))


@pytest.mark.parametrize("sc", [_drop_stack(TINY, 0.2, 0xFEDCBA9876543210), _drop_stack(TINY_TIED, 0.1, 12)])
def test_stack_with_dropout_against_torch_autograd(sc):
    w, tokens, targets = _stack_case(sc)
    loss, saved = O.stack_loss(sc, tokens, targets, w)
    g = O.stack_loss_grad(sc, w, saved)
    tw = _to_torch(w)
    tl = _torch_stack_loss_drop(sc, tokens, targets, tw)
    tl.backward()
    assert abs(loss - float(tl.detach())) < 1e-12 * max(1.0, abs(loss))
    scale = lambda a: np.sqrt(np.mean(a * a)) + 1e-300
    for name in ["embedding", "rel_table", "final_scale"] + ([] if sc.tied_logits else ["logits_w"]):
        ref = tw[name].grad.numpy()
        assert np.abs(g[name] - ref).max() / scale(ref) < 1e-9, name
    for l in range(sc.n_layers):
        for name, val in g["layers"][l].items():
            ref = tw["layers"][l][name].grad.numpy()
            assert np.abs(val - ref).max() / scale(ref) < 1e-9, (l, name)
    # the layers do not share masks, and rate 0 is the plain stack bit for bit
    m0, m1 = saved["layers"][0]["drop"], saved["layers"][1]["drop"]
    assert all(not np.array_equal(m0[s], m1[s]) for s in (1, 2, 3, 4))
    plain = replace(sc, block=replace(sc.block, dropout_rate=0.0, dropout_seed=0))
    assert O.stack_loss(_drop_stack(sc, 0.0, 99), tokens, targets, w)[0] == O.stack_loss(plain, tokens, targets, w)[0]
    assert abs(O.stack_loss(plain, tokens, targets, w)[0] - loss) > 1e-4


def _torch_encdec_loss_drop(ec, enc_tokens, dec_tokens, targets, tw):
    e, d = ec.enc_block, ec.dec_block
    B, dm = e.batch, e.d_model
    tm = lambda cfg, site, S: torch.from_numpy(_mask(cfg.dropout_seed, site, B * S, dm, cfg.dropout_rate, (B, S, dm)))
    x = tw["embedding"][torch.from_numpy(enc_tokens).long()] * tm(e, 7, e.seq)
    for l, lw in enumerate(tw["enc_layers"]):
        x = _torch_block_drop(e, x, dict(lw, rel_table=tw["enc_rel_table"]),
                              _block_masks(e, (e.dropout_seed + (l + 1) * GOLD) & M64))
    enc_out = F.rms_norm(x, (dm,), tw["enc_final_scale"], eps=e.rms_eps) * tm(e, 8, e.seq)
    x = tw["embedding"][torch.from_numpy(dec_tokens).long()] * tm(d, 9, d.seq)
    for l, lw in enumerate(tw["dec_layers"]):
        seed_l = (d.dropout_seed + (ec.n_enc_layers + l + 1) * GOLD) & M64
        x = _torch_decoder_block_drop(d, x, enc_out, dict(lw, rel_table=tw["dec_rel_table"]),
                                      _decoder_masks(d, seed_l, e.seq))
    nf = F.rms_norm(x, (dm,), tw["dec_final_scale"], eps=d.rms_eps) * tm(d, 10, d.seq)
    logits = (nf * dm ** -0.5) @ tw["embedding"].T if ec.tied_logits else nf @ tw["logits_w"]
    tt = torch.from_numpy(targets).long()
    valid = tt >= 0
    lse = torch.logsumexp(logits, -1)
    ce = F.cross_entropy(logits.reshape(-1, ec.vocab), tt.reshape(-1), ignore_index=-1, reduction="sum")
    return (ce + ec.z_loss * (lse[valid] ** 2).sum()) / valid.sum()


def _drop_encdec(ec, rate, seed_e, seed_d):
    return replace(ec, enc_block=replace(ec.enc_block, dropout_rate=rate, dropout_seed=seed_e),
                   dec_block=replace(ec.dec_block, dropout_rate=rate, dropout_seed=seed_d))


@pytest.mark.parametrize("ec", [_drop_encdec(EC, 0.15, 0x1111222233334444, 0x1111222233334444),
                                _drop_encdec(EC_TIED, 0.3, 5, 6)])
def test_encdec_with_dropout_against_torch_autograd(ec):
    w, enc_tokens, dec_tokens, targets = _ec_case(ec)
    loss, saved = O.encdec_loss(ec, enc_tokens, dec_tokens, targets, w)
    g = O.encdec_loss_grad(ec, w, saved)
    tw = _to_torch(w)
    tl = _torch_encdec_loss_drop(ec, enc_tokens, dec_tokens, targets, tw)
    tl.backward()
    assert abs(loss - float(tl.detach())) < 1e-12 * max(1.0, abs(loss))
    scale = lambda a: np.sqrt(np.mean(a * a)) + 1e-300
    for name in [k for k in w if not k.endswith("_layers")]:
        ref = tw[name].grad.numpy()
        assert np.abs(g[name] - ref).max() / scale(ref) < 1e-9, name
    for side in ("enc_layers", "dec_layers"):
        for l, lw in enumerate(w[side]):
            for name, val in g[side][l].items():
                ref = tw[side][l][name].grad.numpy()
                assert np.abs(val - ref).max() / scale(ref) < 1e-9, (side, l, name)


def test_stack_dropout_gradients_against_central_differences():
    sc = _drop_stack(TINY, 0.2, 77)
    w, tokens, targets = _stack_case(sc)
    loss, saved = O.stack_loss(sc, tokens, targets, w)
    g = O.stack_loss_grad(sc, w, saved)
    f = lambda: O.stack_loss(sc, tokens, targets, w)[0]
    rng = np.random.default_rng(5)
    eps = 1e-6
    for arr, grad, name in ((w["embedding"], g["embedding"], "embedding"), (w["final_scale"], g["final_scale"], "final"),
                            (w["layers"][1]["wo"], g["layers"][1]["wo"], "wo1"),
                            (w["layers"][0]["wi0"], g["layers"][0]["wi0"], "wi0_0"), (w["rel_table"], g["rel_table"], "tab")):
        for fi in rng.choice(arr.size, size=4, replace=False):
            idx = np.unravel_index(fi, arr.shape)
            old = arr[idx]
            arr[idx] = old + eps; lp = f()
            arr[idx] = old - eps; lm = f()
            arr[idx] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad[idx]) <= 2e-6 * max(1.0, abs(grad[idx])), (name, idx, fd, grad[idx])
