"""Pins for the oracle's dropout (CPU only): the counter-based generator's structural and statistical
properties, and the block's forward/backward with the masks against torch autograd and finite differences."""
from dataclasses import replace
import math

import numpy as np
import pytest
import torch

import synth_inputs as SI
from oracle import t5_oracle as O
from test_oracle_block import TINY, TINY_CAUSAL, _case, _torch_mlp, _bucket_from_fixture
import torch.nn.functional as F


def _mix32_int(x: int) -> int:
    """The finaliser on Python integers (arbitrary precision, reduced by hand), independent of numpy's
    fixed-width arithmetic."""
    x &= 0xFFFFFFFF
    x ^= x >> 16
    x = (x * 0x7FEB352D) % (1 << 32)
    x ^= x >> 15
    x = (x * 0x846CA68B) % (1 << 32)
    x ^= x >> 16
    return x


def test_generator_matches_big_integer_evaluation_elementwise():
    seed, site, rate = 0x1234ABCD9876EF01, 3, 0.3
    keep = O.dropout_keep(seed, site, 40, 70, rate)
    k0 = _mix32_int((seed & 0xFFFFFFFF) ^ ((site * 0x9E3779B9) % (1 << 32)))
    thr = math.floor(rate * 2 ** 32)
    for hi, lo in [(0, 0), (1, 0), (0, 1), (39, 69), (17, 33), (5, 64)]:
        r = _mix32_int(_mix32_int(k0 ^ hi ^ (seed >> 32)) ^ lo)
        assert bool(keep[hi, lo]) == (r >= thr), (hi, lo)
    # the finaliser is a bijection on 32 bits (xor-shifts and odd multiplications are invertible):
    # no two of many inputs collide
    xs = np.arange(1 << 16, dtype=np.uint64) * np.uint64(65537)
    assert len(np.unique(O._mix32(xs))) == len(xs)


def test_generator_is_stateless_and_tiling_independent():
    a = O.dropout_keep(77, 1, 64, 96, 0.25)
    b = O.dropout_keep(77, 1, 200, 300, 0.25)
    assert np.array_equal(a, b[:64, :96])                  # an element depends on its indices only
    assert np.array_equal(a, O.dropout_keep(77, 1, 64, 96, 0.25))
    # a larger rate drops a superset (the threshold moves, the random word does not)
    c = O.dropout_keep(77, 1, 64, 96, 0.5)
    assert np.all(a[c])                                    # kept at 0.5 implies kept at 0.25
    assert O.dropout_keep(77, 1, 8, 8, 0.0).all()


@pytest.mark.parametrize("rate", [0.1, 0.5])
def test_generator_statistics(rate):
    n_hi, n_lo = 512, 2048
    k = O.dropout_keep(20220331, 2, n_hi, n_lo, rate)
    n = n_hi * n_lo
    sd = math.sqrt(rate * (1 - rate) / n)
    assert abs(k.mean() - (1 - rate)) < 5 * sd
    # rows and columns individually
    assert np.abs(k.mean(1) - (1 - rate)).max() < 6 * math.sqrt(rate * (1 - rate) / n_lo)
    assert np.abs(k.mean(0) - (1 - rate)).max() < 6 * math.sqrt(rate * (1 - rate) / n_hi)
    # neighbours, other sites and other seeds are uncorrelated with it
    x = k.astype(np.float64) - (1 - rate)
    var = rate * (1 - rate)
    for other in (np.roll(x, 1, axis=1), np.roll(x, 1, axis=0),
                  O.dropout_keep(20220331, 3, n_hi, n_lo, rate) - (1 - rate),
                  O.dropout_keep(20220332, 2, n_hi, n_lo, rate) - (1 - rate),
                  O.dropout_keep(20220331 + (1 << 32), 2, n_hi, n_lo, rate) - (1 - rate)):
        assert abs(np.mean(x * other)) / var < 6 / math.sqrt(n)


DROP = replace(TINY, name="tiny_drop", index=30, dropout_rate=0.2, dropout_seed=0xC0FFEE1234)
DROP_CAUSAL_RELU = replace(TINY_CAUSAL, name="tiny_drop_relu", index=31, dropout_rate=0.35, dropout_seed=99, mlp="relu")


def _torch_block_drop(cfg, x, w, drop):
    B, S, H, K = cfg.batch, cfg.seq, cfg.n_heads, cfg.d_kv
    m = {k: torch.from_numpy(v) for k, v in drop.items()}
    n1 = F.rms_norm(x, (cfg.d_model,), w["ln1_scale"], eps=cfg.rms_eps)
    heads = lambda t, mm: torch.einsum("bsd,dhk->bhsk", t, mm.view(cfg.d_model, H, K))
    q, k, v = heads(n1, w["wq"]), heads(n1, w["wk"]), heads(n1, w["wv"])
    idx = torch.tensor([[_bucket_from_fixture(j - i, cfg.causal) for j in range(S)] for i in range(S)])
    logits = cfg.attn_scale * torch.einsum("bhik,bhjk->bhij", q, k) + w["rel_table"][idx].permute(2, 0, 1)
    if cfg.causal:
        logits = logits.masked_fill(~torch.ones(S, S, dtype=torch.bool).tril(), float("-inf"))
    p = F.softmax(logits, dim=-1) * m[O.DROP_ATTN_PROBS]
    o = torch.einsum("bhij,bhjk->bihk", p, v).reshape(B, S, H * K)
    h = x + (o @ w["wo"]) * m[O.DROP_ATTN_OUT]
    n2 = F.rms_norm(h, (cfg.d_model,), w["ln2_scale"], eps=cfg.rms_eps)
    if cfg.mlp == "relu":
        a = F.relu(n2 @ w["wi0"])
    else:
        a = F.gelu(n2 @ w["wi0"], approximate="tanh") * (n2 @ w["wi1"])
    return h + ((a * m[O.DROP_MLP_HIDDEN]) @ w["wo_ff"]) * m[O.DROP_MLP_OUT]


@pytest.mark.parametrize("cfg", [DROP, DROP_CAUSAL_RELU])
def test_block_with_dropout_against_torch_autograd(cfg):
    w, x, dy = _case(cfg)
    y, saved = O.block_fwd(cfg, x, w)
    dx, g = O.block_bwd(cfg, dy, w, saved)
    assert saved["drop"] is not None
    tw = {k_: torch.from_numpy(np.ascontiguousarray(v)).requires_grad_() for k_, v in w.items()}
    tx = torch.from_numpy(x).requires_grad_()
    ty = _torch_block_drop(cfg, tx, tw, saved["drop"])
    ty.backward(torch.from_numpy(dy))
    np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-11, atol=1e-12)
    scale = lambda a: np.sqrt(np.mean(a * a)) + 1e-300
    assert np.abs(dx - tx.grad.numpy()).max() / scale(dx) < 1e-10
    for name, val in g.items():
        assert np.abs(val - tw[name].grad.numpy()).max() / scale(val) < 1e-10, name


def test_block_dropout_structure():
    w, x, dy = _case(DROP)
    y, saved = O.block_fwd(DROP, x, w)
    d = saved["drop"]
    keep = 1.0 - DROP.dropout_rate
    for site, shape in ((O.DROP_ATTN_PROBS, (2, 2, 12, 12)), (O.DROP_ATTN_OUT, (2, 12, 16)),
                        (O.DROP_MLP_HIDDEN, (2, 12, 24)), (O.DROP_MLP_OUT, (2, 12, 16))):
        assert d[site].shape == shape
        assert set(np.unique(d[site])) <= {0.0, 1.0 / keep}
    # the four sites use different masks
    assert not np.array_equal(d[O.DROP_ATTN_OUT], d[O.DROP_MLP_OUT])
    # attention rows: the probabilities that multiply v are the softmax times the mask (they no longer sum to 1)
    np.testing.assert_allclose(saved["pd"], saved["p"] * d[O.DROP_ATTN_PROBS], rtol=0, atol=0)
    # rate 0 is the plain block, bit for bit; another seed gives another output
    y0, s0 = O.block_fwd(replace(DROP, dropout_rate=0.0), x, w)
    yp, _ = O.block_fwd(replace(DROP, dropout_rate=0.0, dropout_seed=5), x, w)
    assert s0["drop"] is None and np.array_equal(y0, yp)
    y2, _ = O.block_fwd(replace(DROP, dropout_seed=DROP.dropout_seed + 1), x, w)
    assert np.abs(y2 - y).max() > 1e-3
    # dropping everything but the residual: with the two output masks forced to zero y = x
    # (checked through the backward: no gradient reaches the weights when every site output is dropped)


def test_block_dropout_backward_against_central_differences():
    cfg = DROP
    w, x, dy = _case(cfg)
    y, saved = O.block_fwd(cfg, x, w)
    dx, g = O.block_bwd(cfg, dy, w, saved)
    loss = lambda xx, ww: float(np.sum(O.block_fwd(cfg, xx, ww)[0] * dy))
    rng = np.random.default_rng(3)
    eps = 1e-6
    for name in ("x", "wq", "wv", "wo", "wi0", "wi1", "wo_ff", "rel_table", "ln1_scale", "ln2_scale"):
        arr = x if name == "x" else w[name]
        grad = dx if name == "x" else g[name]
        for fi in rng.choice(arr.size, size=5, replace=False):
            idx = np.unravel_index(fi, arr.shape)
            old = arr[idx]
            arr[idx] = old + eps; lp = loss(x, w)
            arr[idx] = old - eps; lm = loss(x, w)
            arr[idx] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad[idx]) <= 2e-6 * max(1.0, abs(grad[idx])), (name, idx, fd, grad[idx])
