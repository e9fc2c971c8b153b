"""GPU parity of the decoder layer (causal self-attention, cross-attention over an encoder output,
MLP) through the C ABI against the float64 oracle, element by element."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import synth_inputs as SI
from oracle import t5_oracle as O
from parity_util import (TOL_F32, check_bf16, decoder_floors, is_relu, make_decoder_case, rel_err,
                         run_decoder_block_gpu, to_dev, to_np)

pytestmark = pytest.mark.gpu

C1 = SI.CONFIGS["c1_tiny_f32"]
F32_CASES = [
    replace(C1, name="dec_f32", index=40, causal=True, enc_seq=48),
    replace(C1, name="dec_f32_ragged", index=41, batch=3, seq=37, d_model=72, n_heads=3, d_kv=20, d_ff=100,
            attn_scale=0.25, causal=True, enc_seq=53),
    replace(C1, name="dec_f32_one_enc_token", index=42, causal=True, enc_seq=1),
    replace(C1, name="dec_f32_long_enc", index=43, batch=1, seq=20, causal=True, enc_seq=300),
    replace(C1, name="dec_f32_bidirectional_self", index=44, causal=False, enc_seq=70),
    replace(C1, name="dec_f32_relu", index=51, causal=True, enc_seq=48, mlp="relu"),
]


def _check_bf16(cfg):
    """bf16 decoder layer against the oracle, every tensor at the bound derived from its ideal-bf16 floor."""
    w, x, enc, dy = make_decoder_case(cfg)
    y, saved = O.decoder_block_fwd(cfg, x, enc, w)
    dx, denc, g = O.decoder_block_bwd(cfg, dy, w, saved)
    gy, gdx, gdenc, gg = run_decoder_block_gpu(cfg, w, x, enc, dy)
    assert set(gg) == set(g)
    errs = {"y": rel_err(gy, y), "dx": rel_err(gdx, dx), "denc": rel_err(gdenc, denc),
            **{k: rel_err(gg[k], g[k]) for k in g}}
    check_bf16(cfg.name, errs, decoder_floors(cfg, w, x, enc, dy, (y, dx, denc, g)), relu=is_relu(cfg))


def _check(cfg, tol_y, tol_dx, tol_denc, tol_dw, verbose=True):
    w, x, enc, dy = make_decoder_case(cfg)
    y, saved = O.decoder_block_fwd(cfg, x, enc, w)
    dx, denc, g = O.decoder_block_bwd(cfg, dy, w, saved)
    gy, gdx, gdenc, gg = run_decoder_block_gpu(cfg, w, x, enc, dy)
    ey, edx, ede = rel_err(gy, y), rel_err(gdx, dx), rel_err(gdenc, denc)
    if verbose:
        print(cfg.name, "y", ey, "dx", edx, "denc", ede, {k: tuple(round(v, 5) for v in rel_err(gg[k], g[k])) for k in g})
    assert ey[0] <= tol_y[0] and ey[1] <= tol_y[1], ("y", ey)
    assert edx[0] <= tol_dx[0] and edx[1] <= tol_dx[1], ("dx", edx)
    assert ede[0] <= tol_denc[0] and ede[1] <= tol_denc[1], ("denc", ede)
    assert set(gg) == set(g)
    for name in g:
        e = rel_err(gg[name], g[name])
        assert e[0] <= tol_dw[0] and e[1] <= tol_dw[1], (name, e)


@pytest.mark.parametrize("cfg", F32_CASES, ids=[c.name for c in F32_CASES])
def test_decoder_block_f32(cfg):
    _check(cfg, TOL_F32, TOL_F32, TOL_F32, TOL_F32)


SMALL_BF16 = [
    # MFMA attention both ways (sequence lengths multiples of 128), decoder shorter than encoder and longer
    SI.BlockConfig("dec_bf16", 45, batch=2, seq=128, d_model=128, n_heads=2, d_kv=64, d_ff=256, causal=True,
                   attn_scale=64 ** -0.5, enc_seq=256),
    SI.BlockConfig("dec_bf16_long_dec", 46, batch=2, seq=384, d_model=128, n_heads=2, d_kv=64, d_ff=256, causal=True,
                   attn_scale=64 ** -0.5, enc_seq=128),
    SI.BlockConfig("dec_bf16_dk128", 47, batch=1, seq=256, d_model=256, n_heads=2, d_kv=128, d_ff=320, causal=True,
                   attn_scale=128 ** -0.5, enc_seq=384),
    # three heads: workgroups are not dealt in groups of eight
    SI.BlockConfig("dec_bf16_h3", 48, batch=1, seq=128, d_model=192, n_heads=3, d_kv=64, d_ff=192, causal=True,
                   attn_scale=64 ** -0.5, enc_seq=128),
    # encoder length not a multiple of the attention tiles: ragged key tiles in the fused cross-attention
    SI.BlockConfig("dec_bf16_ragged_enc", 49, batch=2, seq=128, d_model=128, n_heads=2, d_kv=64, d_ff=256, causal=True,
                   attn_scale=64 ** -0.5, enc_seq=100),
    # T5's own lengths: 114 decoder positions over 512 encoder positions, and a ragged pair
    SI.BlockConfig("dec_bf16_s114", 53, batch=2, seq=114, d_model=128, n_heads=2, d_kv=64, d_ff=256, causal=True,
                   attn_scale=64 ** -0.5, enc_seq=512),
    SI.BlockConfig("dec_bf16_s200_e77", 54, batch=1, seq=200, d_model=128, n_heads=2, d_kv=128, d_ff=256, causal=True,
                   attn_scale=128 ** -0.5, enc_seq=77),
    SI.BlockConfig("dec_bf16_relu", 52, batch=2, seq=128, d_model=128, n_heads=2, d_kv=64, d_ff=256, causal=True,
                   attn_scale=64 ** -0.5, enc_seq=128, mlp="relu"),
    # nothing a multiple of anything: simple kernels throughout
    SI.BlockConfig("dec_bf16_ragged", 50, batch=1, seq=100, d_model=72, n_heads=3, d_kv=24, d_ff=136, causal=True,
                   attn_scale=24 ** -0.5, enc_seq=61),
]


def test_ragged_lengths_run_the_fused_attention_kernels():
    import paper_2203_17189_amd as P
    want = P.PATH_MFMA_ATTN_FWD | P.PATH_MFMA_ATTN_BWD | P.PATH_MFMA_CROSS_ATTN
    for cfg in SMALL_BF16:
        if cfg.d_kv in (64, 128):
            assert P.t5_block_kernel_path(cfg) & want == want, (cfg.name, P.t5_block_kernel_path(cfg))
    assert P.t5_block_kernel_path(SMALL_BF16[-1]) & want == 0      # 24 channels per head: general-shape kernels


@pytest.mark.parametrize("cfg", SMALL_BF16, ids=[c.name for c in SMALL_BF16])
def test_decoder_block_bf16_small(cfg):
    _check_bf16(cfg)


def test_decoder_named_config_reduced_batch():
    """T5.1.1-Base decoder layer at its real widths and lengths, batch reduced for the oracle."""
    cfg = replace(SI.CONFIGS["c6_dec_base"], attn_scale=64 ** -0.5).with_batch(2)
    _check_bf16(cfg)


def test_decoder_named_config_full_batch_sampled():
    """c6_dec_base at its full batch, as bench.py launches it: the first sequence's y, dx and denc against the
    oracle (sequences, each with its own encoder output, are independent through the layer)."""
    import paper_2203_17189_amd as P
    cfg = replace(SI.CONFIGS["c6_dec_base"], attn_scale=64 ** -0.5)
    w, x, enc, dy = make_decoder_case(cfg)
    small = cfg.with_batch(1)
    y, saved = O.decoder_block_fwd(small, x[:1], enc[:1], w)
    dx, denc, g_small = O.decoder_block_bwd(small, dy[:1], w, saved)
    dw = {k: to_dev(v, cfg.dtype) for k, v in w.items()}
    tx, te, tdy = to_dev(x, cfg.dtype), to_dev(enc, cfg.dtype), to_dev(dy, cfg.dtype)
    gy, stash = P.t5_decoder_block_fwd(cfg, tx, te, dw)
    gdx, gdenc, gg = P.t5_decoder_block_bwd(cfg, tdy, tx, te, dw, stash)
    torch.cuda.synchronize()
    errs = {"y": rel_err(to_np(gy[:1]), y), "dx": rel_err(to_np(gdx[:1]), dx), "denc": rel_err(to_np(gdenc[:1]), denc)}
    check_bf16("c6_dec_base full batch sample", errs,
               decoder_floors(small, w, x[:1], enc[:1], dy[:1], (y, dx, denc, g_small)), only=("y", "dx", "denc"))
    assert all(torch.isfinite(v).all() for v in gg.values())


def test_decoder_accumulate_and_determinism():
    import paper_2203_17189_amd as P
    cfg = SMALL_BF16[0]
    w, x, enc, dy = make_decoder_case(cfg)
    dw = {k: to_dev(v, cfg.dtype) for k, v in w.items()}
    tx, te, tdy = to_dev(x, cfg.dtype), to_dev(enc, cfg.dtype), to_dev(dy, cfg.dtype)
    y, stash = P.t5_decoder_block_fwd(cfg, tx, te, dw)
    dx, denc, g1 = P.t5_decoder_block_bwd(cfg, tdy, tx, te, dw, stash)
    g2 = {k: v.clone() for k, v in g1.items()}
    dx2, denc2, _ = P.t5_decoder_block_bwd(cfg, tdy, tx, te, dw, stash, grads=g2, accumulate=True)
    torch.cuda.synchronize()
    assert torch.equal(dx, dx2) and torch.equal(denc, denc2)       # no atomics on the activation gradients
    for k in g1:
        a1 = to_np(g1[k])
        scale = np.abs(a1).max() + 1e-30
        assert np.abs(to_np(g2[k]) - 2 * a1).max() <= 4e-5 * scale, ("accumulate", k)


def test_decoder_encoder_tokens_form_a_set():
    """Permuting the encoder tokens leaves y unchanged and permutes denc the same way (cross-attention
    carries no positions).  The two runs differ in summation order, which moves bf16 roundings of the
    stored intermediates, so they are compared at the bounds used against the oracle."""
    cfg = SMALL_BF16[0]
    w, x, enc, dy = make_decoder_case(cfg)
    perm = np.random.default_rng(3).permutation(cfg.enc_seq)
    y1, dx1, de1, g1 = run_decoder_block_gpu(cfg, w, x, enc, dy)
    y2, dx2, de2, g2 = run_decoder_block_gpu(cfg, w, x, enc[:, perm], dy)
    errs = {"y": rel_err(y2, y1), "denc": rel_err(de2, de1[:, perm])}
    floors = decoder_floors(cfg, w, x, enc, dy, None)
    check_bf16(cfg.name + " permuted encoder", errs, floors, scale=2 ** 0.5, only=("y", "denc"))
    # and the unpermuted comparison is far outside them, so the check can tell the two apart
    assert rel_err(de2, de1)[1] > 10 * 1.25 * floors["denc"][1]
