"""Pins for the oracle's block forward/backward (CPU only).

Each test ties the oracle to something other than itself: a library routine
(torch's scaled_dot_product_attention, rms_norm, tanh-GELU, autograd), a closed
form, an invariant of the mathematics, or finite differences.
"""
from dataclasses import replace

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as SI
from conftest import read_golden_pairs
from oracle import t5_oracle as O

TINY = SI.BlockConfig("tiny", 9, batch=2, seq=12, d_model=16, n_heads=2, d_kv=4, d_ff=24, dtype="f32")
TINY_CAUSAL = replace(TINY, name="tiny_causal", index=10, causal=True, attn_scale=0.5)


def _case(cfg, random_scales=True):
    w = SI.make_weights(cfg)
    if random_scales:
        w.update(SI.make_random_scales(cfg))
    x, dy = SI.make_activations(cfg)
    return w, x, dy


# ---------------------------------------------------------------- softmax / attention
@pytest.mark.parametrize("cfg", [TINY, TINY_CAUSAL, SI.CONFIGS["c1_tiny_f32"]])
def test_softmax_rows_sum_to_one(cfg):
    w, x, _ = _case(cfg)
    _, saved = O.block_fwd(cfg, x, w)
    p = saved["p"]
    assert np.all(p >= 0)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=0, atol=1e-14)
    if cfg.causal:
        iu = np.triu_indices(cfg.seq, 1)
        assert np.all(p[..., iu[0], iu[1]] == 0.0)


@pytest.mark.parametrize("causal", [False, True])
def test_reduces_to_library_scaled_dot_product_attention(causal):
    """Zero bias table and attn_scale = d_kv^-1/2 is textbook attention: compare the merged head
    outputs with torch's library routine in float64."""
    cfg = replace(TINY, causal=causal, attn_scale=TINY.d_kv ** -0.5)
    w, x, _ = _case(cfg)
    w["rel_table"] = np.zeros_like(w["rel_table"])
    _, saved = O.block_fwd(cfg, x, w)
    tq, tk, tv = (torch.from_numpy(saved[n]) for n in ("q", "k", "v"))
    ref = F.scaled_dot_product_attention(tq, tk, tv, is_causal=causal)          # [B,H,S,k]
    ref = ref.permute(0, 2, 1, 3).reshape(cfg.batch, cfg.seq, cfg.inner).numpy()
    np.testing.assert_allclose(saved["c"], ref, rtol=1e-12, atol=1e-13)


def test_head_split_matches_column_blocks():
    """Column h*d_kv + c of Wq belongs to head h: check q of head 1 against a direct product."""
    w, x, _ = _case(TINY)
    _, saved = O.block_fwd(TINY, x, w)
    k_ = TINY.d_kv
    direct = saved["n1"] @ w["wq"][:, k_:2 * k_]
    np.testing.assert_allclose(saved["q"][:, 1], direct, rtol=1e-13, atol=1e-14)


def test_table_shift_invariance_and_bias_effect():
    w, x, _ = _case(TINY)
    y0, _ = O.block_fwd(TINY, x, w)
    w2 = dict(w)
    w2["rel_table"] = w["rel_table"] + np.array([[0.7, -1.3]])   # constant per head
    y1, _ = O.block_fwd(TINY, x, w2)
    np.testing.assert_allclose(y1, y0, rtol=1e-12, atol=1e-12)
    w3 = dict(w)
    t3 = w["rel_table"].copy()
    t3[1, 0] += 2.0                                              # bucket 1 = key just before query
    w3["rel_table"] = t3
    y3, s3 = O.block_fwd(TINY, x, w3)
    assert np.abs(y3 - y0).max() > 1e-3
    _, s0 = O.block_fwd(TINY, x, w)
    # head 0 now attends more to key i-1, head 1 is untouched
    i = np.arange(1, TINY.seq)
    assert np.all(s3["p"][:, 0, i, i - 1] > s0["p"][:, 0, i, i - 1])
    np.testing.assert_array_equal(s3["p"][:, 1], s0["p"][:, 1])


def test_constant_table_bidirectional_is_permutation_equivariant():
    cfg = TINY
    w, x, _ = _case(cfg)
    w["rel_table"] = np.full_like(w["rel_table"], 0.3)
    perm = np.random.default_rng(0).permutation(cfg.seq)
    y, _ = O.block_fwd(cfg, x, w)
    yp, _ = O.block_fwd(cfg, x[:, perm], w)
    np.testing.assert_allclose(yp, y[:, perm], rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- causal
def test_causal_outputs_ignore_future_tokens():
    cfg = TINY_CAUSAL
    w, x, dy = _case(cfg)
    y0, _ = O.block_fwd(cfg, x, w)
    i0 = 7
    x2 = x.copy()
    x2[:, i0 + 1:] += np.random.default_rng(1).standard_normal(x2[:, i0 + 1:].shape)
    y1, _ = O.block_fwd(cfg, x2, w)
    assert np.array_equal(y1[:, :i0 + 1], y0[:, :i0 + 1])          # bit-unchanged
    assert np.abs(y1[:, i0 + 1:] - y0[:, i0 + 1:]).max() > 1e-3
    # gradient side: dy supported on positions < i0 gives no gradient to positions >= i0
    dy2 = dy.copy()
    dy2[:, i0:] = 0.0
    y, saved = O.block_fwd(cfg, x, w)
    dx, _ = O.block_bwd(cfg, dy2, w, saved)
    assert np.all(dx[:, i0:] == 0.0)
    assert np.abs(dx[:, :i0]).min() > 0.0


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_against_library_and_invariants():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((3, 7, 24))
    g = 1.0 + 0.2 * rng.standard_normal(24)
    n, r = O.rmsnorm_fwd(x, g, 1e-6)
    ref = F.rms_norm(torch.from_numpy(x), (24,), torch.from_numpy(g), eps=1e-6).numpy()
    np.testing.assert_allclose(n, ref, rtol=1e-13, atol=1e-14)
    # positive scaling invariance is exact when eps = 0
    n0, _ = O.rmsnorm_fwd(x, g, 0.0)
    n1, _ = O.rmsnorm_fwd(3.7 * x, g, 0.0)
    np.testing.assert_allclose(n1, n0, rtol=1e-14, atol=1e-15)
    # ||x r||^2 = d (1 - eps r^2)
    xh = x * r
    np.testing.assert_allclose((xh * xh).sum(-1, keepdims=True), 24 * (1 - 1e-6 * r * r), rtol=1e-12)
    # no mean subtraction: a constant vector keeps its sign and magnitude 1
    c = np.full((1, 24), 5.0)
    nc, _ = O.rmsnorm_fwd(c, np.ones(24), 0.0)
    np.testing.assert_allclose(nc, 1.0, rtol=1e-14)


def test_rmsnorm_backward_orthogonality_and_autograd():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((5, 16))
    g = 1.0 + 0.2 * rng.standard_normal(16)
    dn = rng.standard_normal((5, 16))
    _, r = O.rmsnorm_fwd(x, g, 0.0)
    dx, dg = O.rmsnorm_bwd(x, g, r, dn)
    # with eps = 0 the input gradient is orthogonal to x (scaling x does not change the output)
    np.testing.assert_allclose((dx * x).sum(-1), 0.0, atol=1e-13)
    tx = torch.from_numpy(x).requires_grad_()
    tg = torch.from_numpy(g).requires_grad_()
    F.rms_norm(tx, (16,), tg, eps=0.0).backward(torch.from_numpy(dn))
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dg, tg.grad.numpy(), rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- MLP / GELU
def test_gelu_against_library_and_identities():
    z = np.linspace(-9, 9, 2001)
    ref = F.gelu(torch.from_numpy(z), approximate="tanh").numpy()
    np.testing.assert_allclose(O.gelu(z), ref, rtol=1e-13, atol=1e-15)
    assert O.gelu(np.array(0.0)) == 0.0 and O.gelu_grad(np.array(0.0)) == 0.5
    np.testing.assert_allclose(O.gelu(z) - O.gelu(-z), z, rtol=0, atol=1e-14)     # tanh is odd
    np.testing.assert_allclose(O.gelu(np.array([30.0, -30.0])), [30.0, 0.0], atol=1e-12)
    tz = torch.from_numpy(z).requires_grad_()
    F.gelu(tz, approximate="tanh").sum().backward()
    np.testing.assert_allclose(O.gelu_grad(z), tz.grad.numpy(), rtol=1e-12, atol=1e-14)


def test_gate_order_wi0_goes_through_gelu():
    cfg = TINY
    w, x, _ = _case(cfg)
    _, saved = O.block_fwd(cfg, x, w)
    n2 = saved["n2"]
    want = F.gelu(torch.from_numpy(n2 @ w["wi0"]), approximate="tanh").numpy() * (n2 @ w["wi1"])
    np.testing.assert_allclose(saved["a"], want, rtol=1e-12, atol=1e-14)


def test_zero_output_projections_give_identity():
    cfg = TINY
    w, x, dy = _case(cfg)
    w["wo"] = np.zeros_like(w["wo"])
    w["wo_ff"] = np.zeros_like(w["wo_ff"])
    y, saved = O.block_fwd(cfg, x, w)
    assert np.array_equal(y, x)
    dx, g = O.block_bwd(cfg, dy, w, saved)
    assert np.array_equal(dx, dy)
    assert np.abs(g["wo"]).max() > 0 and np.abs(g["wo_ff"]).max() > 0
    for name in ("wq", "wk", "wv", "wi0", "wi1", "rel_table", "ln1_scale", "ln2_scale"):
        assert np.all(g[name] == 0.0), name


# ---------------------------------------------------------------- backward: autograd second opinion
def _first_n_tables():
    bi, uni = {}, {}
    for mode, bucket, first_n in read_golden_pairs("relpos_first_n_32_128.txt"):
        (bi if mode == "bi" else uni)[int(bucket)] = int(first_n)
    return bi, uni


def _bucket_from_fixture(rp, causal):
    """Bucket from the hand-derived 'first n' fixture (independent of the oracle's integer form)."""
    bi, uni = _first_n_tables()
    if causal:
        n = max(-rp, 0)
        if n < 16:
            return n
        return max(b for b, f in uni.items() if f <= n)
    n = abs(rp)
    base = 16 if rp > 0 else 0
    if n < 8:
        return base + n
    return base + max(b for b, f in bi.items() if f <= n)


def _torch_mlp(cfg, n2, w):
    if cfg.mlp == "relu":
        return F.relu(n2 @ w["wi0"]) @ w["wo_ff"]
    approx = "tanh" if cfg.mlp == "geglu_tanh" else "none"
    return (F.gelu(n2 @ w["wi0"], approximate=approx) * (n2 @ w["wi1"])) @ w["wo_ff"]


def _torch_block(cfg, x, w):
    """Independent forward written with torch library ops (einsum, rms_norm, softmax, gelu)."""
    B, S, H, K = cfg.batch, cfg.seq, cfg.n_heads, cfg.d_kv
    n1 = F.rms_norm(x, (cfg.d_model,), w["ln1_scale"], eps=cfg.rms_eps)
    q = torch.einsum("bsd,dhk->bhsk", n1, w["wq"].view(cfg.d_model, H, K))
    k = torch.einsum("bsd,dhk->bhsk", n1, w["wk"].view(cfg.d_model, H, K))
    v = torch.einsum("bsd,dhk->bhsk", n1, w["wv"].view(cfg.d_model, H, K))
    idx = torch.tensor([[_bucket_from_fixture(j - i, cfg.causal) for j in range(S)] for i in range(S)])
    bias = w["rel_table"][idx]                                   # [S,S,H]
    logits = cfg.attn_scale * torch.einsum("bhik,bhjk->bhij", q, k) + bias.permute(2, 0, 1)
    if cfg.causal:
        mask = torch.ones(S, S, dtype=torch.bool).tril()
        logits = logits.masked_fill(~mask, float("-inf"))
    p = F.softmax(logits, dim=-1)
    o = torch.einsum("bhij,bhjk->bihk", p, v).reshape(B, S, H * K)
    h = x + o @ w["wo"]
    n2 = F.rms_norm(h, (cfg.d_model,), w["ln2_scale"], eps=cfg.rms_eps)
    return h + _torch_mlp(cfg, n2, w)


@pytest.mark.parametrize("cfg", [TINY, TINY_CAUSAL, SI.CONFIGS["c1_tiny_f32"],
                                 replace(SI.CONFIGS["c1_tiny_f32"], causal=True, seq=160, batch=1, index=11)])
def test_forward_and_backward_against_torch_autograd(cfg):
    w, x, dy = _case(cfg)
    y, saved = O.block_fwd(cfg, x, w)
    dx, g = O.block_bwd(cfg, dy, w, saved)
    tw = {k_: torch.from_numpy(np.ascontiguousarray(v)).requires_grad_() for k_, v in w.items()}
    tx = torch.from_numpy(x).requires_grad_()
    ty = _torch_block(cfg, tx, tw)
    ty.backward(torch.from_numpy(dy))
    np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-11, atol=1e-12)
    scale = lambda a: np.sqrt(np.mean(a * a)) + 1e-300
    assert np.abs(dx - tx.grad.numpy()).max() / scale(dx) < 1e-10
    for name, val in g.items():
        ref = tw[name].grad.numpy()
        assert val.shape == ref.shape
        assert np.abs(val - ref).max() / scale(ref) < 1e-10, name


# ---------------------------------------------------------------- backward: finite differences
@pytest.mark.parametrize("cfg", [TINY, TINY_CAUSAL])
def test_backward_against_central_differences(cfg):
    w, x, dy = _case(cfg)
    y, saved = O.block_fwd(cfg, x, w)
    dx, g = O.block_bwd(cfg, dy, w, saved)
    loss = lambda xx, ww: float(np.sum(O.block_fwd(cfg, xx, ww)[0] * dy))
    rng = np.random.default_rng(17)
    eps = 1e-6

    def check(name, arr, grad, n_probe=12):
        flat_idx = rng.choice(arr.size, size=min(n_probe, arr.size), replace=False)
        for fi in flat_idx:
            idx = np.unravel_index(fi, arr.shape)
            ap, am = arr.copy(), arr.copy()
            ap[idx] += eps
            am[idx] -= eps
            if name == "x":
                fd = (loss(ap, w) - loss(am, w)) / (2 * eps)
            else:
                wp, wm = dict(w), dict(w)
                wp[name], wm[name] = ap, am
                fd = (loss(x, wp) - loss(x, wm)) / (2 * eps)
            assert abs(fd - grad[idx]) <= 2e-6 * max(1.0, abs(grad[idx])), (name, idx, fd, grad[idx])

    check("x", x, dx)
    for name in w:
        check(name, w[name], g[name], n_probe=8 if name != "rel_table" else 64)


@pytest.mark.parametrize("cfg", [TINY, TINY_CAUSAL])
def test_bias_table_gradient_sums_to_zero_per_head(cfg):
    w, x, dy = _case(cfg)
    _, saved = O.block_fwd(cfg, x, w)
    _, g = O.block_bwd(cfg, dy, w, saved)
    assert np.abs(g["rel_table"]).max() > 1e-3
    np.testing.assert_allclose(g["rel_table"].sum(0), 0.0, atol=1e-12)
    if cfg.causal:
        # only buckets reachable with n = i - j < seq get gradient
        reach = set(O.relpos_bucket(-np.arange(cfg.seq), False, 32, 128).tolist())
        for b in range(32):
            if b not in reach:
                assert np.all(g["rel_table"][b] == 0.0)


# ---------------------------------------------------------------- feed-forward variants
TINY_RELU = replace(TINY, name="tiny_relu", index=12, mlp="relu")
TINY_ERF = replace(TINY_CAUSAL, name="tiny_erf", index=13, mlp="geglu_erf")


def test_erf_gelu_against_library_and_identities():
    z = np.linspace(-6, 6, 241)
    tz = torch.from_numpy(z).requires_grad_()
    ty = F.gelu(tz, approximate="none")
    ty.sum().backward()
    np.testing.assert_allclose(O.gelu_erf(z), ty.detach().numpy(), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(O.gelu_erf_grad(z), tz.grad.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(O.gelu_erf(z) - O.gelu_erf(-z), z, rtol=0, atol=1e-14)   # Phi(z) + Phi(-z) = 1
    assert O.gelu_erf(np.array([0.0]))[0] == 0.0 and abs(O.gelu_erf_grad(np.array([0.0]))[0] - 0.5) < 1e-15
    # the tanh form approximates it to a few 1e-4
    assert 1e-5 < np.abs(O.gelu(z) - O.gelu_erf(z)).max() < 1e-3


def test_relu_feed_forward_is_linear_where_all_preactivations_are_positive():
    """Original-T5 feed-forward: with u = n2 Wi0 > 0 everywhere, a = u and the sublayer is the product of
    the two matrices; with u < 0 everywhere it is zero and passes no gradient."""
    cfg = TINY_RELU
    w, x, dy = _case(cfg)
    assert "wi1" not in w
    n2 = np.abs(np.random.default_rng(0).standard_normal((2, 5, cfg.d_model)))
    wpos = dict(w, wi0=np.abs(w["wi0"]))
    out, sv = O.mlp_fwd(cfg, n2, wpos)
    np.testing.assert_allclose(out, n2 @ wpos["wi0"] @ wpos["wo_ff"], rtol=1e-12)
    dn2, g = O.mlp_bwd(cfg, np.ones_like(out), n2, wpos, sv)
    np.testing.assert_allclose(dn2, np.ones_like(out) @ wpos["wo_ff"].T @ wpos["wi0"].T, rtol=1e-12)
    assert set(g) == {"wo_ff", "wi0"}
    wneg = dict(w, wi0=-np.abs(w["wi0"]))
    out, sv = O.mlp_fwd(cfg, n2, wneg)
    dn2, g = O.mlp_bwd(cfg, np.ones_like(out), n2, wneg, sv)
    assert np.all(out == 0) and np.all(dn2 == 0) and np.all(g["wi0"] == 0)


@pytest.mark.parametrize("cfg", [TINY_RELU, TINY_ERF, replace(TINY_RELU, causal=True, index=14)])
def test_variants_forward_and_backward_against_torch_autograd(cfg):
    test_forward_and_backward_against_torch_autograd(cfg)


@pytest.mark.parametrize("cfg", [TINY_RELU, TINY_ERF])
def test_variants_backward_against_central_differences(cfg):
    test_backward_against_central_differences(cfg)
