"""GPU parity of dropout: the keep masks bit for bit against the oracle's generator, and the block's
forward and backward with dropout at its four sites against the float64 oracle."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import synth_inputs as SI
from oracle import t5_oracle as O
from parity_util import (TOL_F32, block_floors, check_bf16, is_relu, make_case, rel_err,
                         run_block_gpu)

pytestmark = pytest.mark.gpu

# the C ABI carries the rate as float32: both sides take the same (float32-representable) number, so that
# floor(rate * 2^32) is one integer
RATE = float(np.float32(0.1))
SEED = 0x9A3C5E7F12345678


def _P():
    import paper_2203_17189_amd as P
    return P


@pytest.mark.parametrize("seed,site,rate,rows,cols", [
    (0, 1, RATE, 7, 5), (SEED, 2, RATE, 300, 129), (SEED, 3, 0.5, 1, 4097), (1 << 63, 4, float(np.float32(0.999)), 65, 64),
    (SEED, 1, 0.0, 33, 17), (12345, 9, float(np.float32(1e-9)), 128, 256)])
def test_dropout_keep_bit_exact(seed, site, rate, rows, cols):
    got = _P().t5_dropout_keep(seed, site, rate, rows, cols).cpu().numpy().astype(bool)
    want = O.dropout_keep(seed, site, rows, cols, rate)
    assert np.array_equal(got, want)


def test_dropout_keep_empty_and_errors():
    P = _P()
    assert P.t5_dropout_keep(1, 1, RATE, 0, 16).numel() == 0
    for bad in (-0.1, 1.0, float("nan")):
        with pytest.raises(P.T5Error):
            P.t5_dropout_keep(1, 1, bad, 4, 4)


C1 = SI.CONFIGS["c1_tiny_f32"]
DROP_F32 = [
    replace(C1, name="drop_enc", index=40, dropout_rate=RATE, dropout_seed=SEED),
    replace(C1, name="drop_dec_ragged", index=41, batch=3, seq=37, d_model=72, n_heads=3, d_kv=20, d_ff=100,
            attn_scale=0.25, causal=True, dropout_rate=float(np.float32(0.3)), dropout_seed=7),
    replace(C1, name="drop_relu", index=42, mlp="relu", dropout_rate=RATE, dropout_seed=SEED + 1),
    replace(C1, name="drop_erf_long", index=43, batch=1, seq=300, mlp="geglu_erf", dropout_rate=RATE,
            dropout_seed=(1 << 64) - 1),
]


@pytest.mark.parametrize("cfg", DROP_F32, ids=[c.name for c in DROP_F32])
def test_block_dropout_f32(cfg):
    w, x, dy = make_case(cfg)
    y, saved = O.block_fwd(cfg, x, w)
    dx, g = O.block_bwd(cfg, dy, w, saved)
    gy, gdx, gg = run_block_gpu(cfg, w, x, dy)
    assert rel_err(gy, y)[0] <= TOL_F32[0], ("y", rel_err(gy, y))
    assert rel_err(gdx, dx)[0] <= TOL_F32[0], ("dx", rel_err(gdx, dx))
    for name in g:
        assert rel_err(gg[name], g[name])[0] <= TOL_F32[0], (name, rel_err(gg[name], g[name]))
    # the masks matter: the same case without dropout is far outside the tolerance
    y0, _ = O.block_fwd(replace(cfg, dropout_rate=0.0), x, w)
    assert rel_err(gy, y0)[0] > 100 * TOL_F32[0]


def test_block_dropout_seed_changes_result_and_repeats():
    P = _P()
    from parity_util import upload_case
    cfg = DROP_F32[0]
    w, x, dy = make_case(cfg)
    dw, dx_in, _ = upload_case(cfg, w, x, dy)
    y1, _ = P.t5_block_fwd(cfg, dx_in, dw)
    y2, _ = P.t5_block_fwd(cfg, dx_in, dw)
    y3, _ = P.t5_block_fwd(replace(cfg, dropout_seed=SEED ^ 1), dx_in, dw)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)
    assert not torch.equal(y1, y3)


DROP_BF16 = [
    SI.BlockConfig("bf16_drop_enc", 44, batch=2, seq=256, d_model=128, n_heads=2, d_kv=64, d_ff=256,
                   attn_scale=64 ** -0.5, dropout_rate=RATE, dropout_seed=SEED),
    SI.BlockConfig("bf16_drop_dec", 45, batch=1, seq=384, d_model=256, n_heads=2, d_kv=128, d_ff=512, causal=True,
                   attn_scale=128 ** -0.5, dropout_rate=RATE, dropout_seed=SEED + 2),
    SI.BlockConfig("bf16_drop_relu", 46, batch=2, seq=128, d_model=128, n_heads=2, d_kv=64, d_ff=256,
                   attn_scale=64 ** -0.5, mlp="relu", dropout_rate=RATE, dropout_seed=SEED + 3),
    SI.BlockConfig("bf16_drop_ragged", 47, batch=1, seq=100, d_model=72, n_heads=3, d_kv=24, d_ff=136, causal=True,
                   attn_scale=24 ** -0.5, dropout_rate=float(np.float32(0.25)), dropout_seed=11),
]


@pytest.mark.parametrize("cfg", DROP_BF16, ids=[c.name for c in DROP_BF16])
def test_block_dropout_bf16(cfg):
    w, x, dy = make_case(cfg)
    y, saved = O.block_fwd(cfg, x, w)
    dx, g = O.block_bwd(cfg, dy, w, saved)
    gy, gdx, gg = run_block_gpu(cfg, w, x, dy)
    errs = {"y": rel_err(gy, y), "dx": rel_err(gdx, dx), **{k: rel_err(gg[k], g[k]) for k in g}}
    # the floor model applies the same masks, so the growth of the error with the rate is part of the floor
    check_bf16(cfg.name, errs, block_floors(cfg, w, x, dy, (y, dx, g)), relu=is_relu(cfg))


# ------------------------------------------------------------------ workload shapes (matrix-unit kernels)
def _named(name, b):
    cfg = SI.CONFIGS[name]
    return replace(cfg, attn_scale=cfg.d_kv ** -0.5, dropout_rate=RATE, dropout_seed=SEED + 5).with_batch(b)


@pytest.mark.parametrize("name,b0", [("c3_base", 2), ("c4_gpt_causal", 1)])
def test_config_dropout_reduced_batch(name, b0):
    """Full sequence length, widths and heads of a workload at a reduced batch (sequences are independent
    through the block): several query and key tiles per head in the fused attention kernels."""
    cfg = _named(name, b0)
    w, x, dy = make_case(cfg)
    y, saved = O.block_fwd(cfg, x, w)
    dx, g = O.block_bwd(cfg, dy, w, saved)
    gy, gdx, gg = run_block_gpu(cfg, w, x, dy)
    errs = {"y": rel_err(gy, y), "dx": rel_err(gdx, dx), **{k: rel_err(gg[k], g[k]) for k in g}}
    check_bf16(name + " dropout", errs, block_floors(cfg, w, x, dy, (y, dx, g)))


def test_dropout_full_batch_sampled():
    """c2_small at its full batch with dropout, as bench.py --dropout launches it: the first 2 sequences of y
    and dx against the oracle (the masks of a sequence depend on its own batch index only), and
    run-to-run determinism."""
    from parity_util import to_dev, to_np
    P = _P()
    cfg = _named("c2_small", SI.CONFIGS["c2_small"].batch)
    b0 = 2
    w = SI.make_weights(cfg)
    x, dy = SI.make_activations(cfg)
    small = cfg.with_batch(b0)
    y, saved = O.block_fwd(small, x[:b0], w)
    dx, g_small = O.block_bwd(small, dy[:b0], w, saved)
    dw = {k: to_dev(v, cfg.dtype) for k, v in w.items()}
    tx, tdy = to_dev(x, cfg.dtype), to_dev(dy, cfg.dtype)
    gy, stash = P.t5_block_fwd(cfg, tx, dw)
    gdx, gg = P.t5_block_bwd(cfg, tdy, tx, dw, stash)
    gy2, stash2 = P.t5_block_fwd(cfg, tx, dw)
    gdx2, _ = P.t5_block_bwd(cfg, tdy, tx, dw, stash2)
    torch.cuda.synchronize()
    errs = {"y": rel_err(to_np(gy[:b0]), y), "dx": rel_err(to_np(gdx[:b0]), dx)}
    check_bf16("c2_small dropout full batch sample", errs,
               block_floors(small, w, x[:b0], dy[:b0], (y, dx, g_small)), only=("y", "dx"))
    assert torch.equal(gy, gy2) and torch.equal(gdx, gdx2)
    assert all(torch.isfinite(v).all() for v in gg.values())


# ------------------------------------------------------------------ decoder layer, stacks, encoder-decoder pair
def _drop_block(cfg, rate=RATE, seed=SEED + 9, **kw):
    return replace(cfg, dropout_rate=rate, dropout_seed=seed, **kw)


def _drop_stack(sc, rate=RATE, seed=SEED + 10, **kw):
    return replace(sc, block=_drop_block(sc.block, rate, seed), **kw)


def _drop_encdec(ec, rate=RATE, seed_e=SEED + 11, seed_d=SEED + 11, **kw):
    return replace(ec, enc_block=_drop_block(ec.enc_block, rate, seed_e), dec_block=_drop_block(ec.dec_block, rate, seed_d), **kw)


def _dec_cases():
    import test_gpu_parity_decoder as TD
    f32 = [_drop_block(TD.F32_CASES[0], name="drop_dec_f32", index=80),
           _drop_block(TD.F32_CASES[1], float(np.float32(0.3)), 5, name="drop_dec_f32_ragged", index=81),
           _drop_block(TD.F32_CASES[5], name="drop_dec_f32_relu", index=82)]
    bf = [_drop_block(c, name="drop_" + c.name, index=83 + i) for i, c in enumerate(TD.SMALL_BF16) if
          c.name in ("dec_bf16", "dec_bf16_dk128", "dec_bf16_ragged_enc", "dec_bf16_ragged")]
    return f32, bf


DEC_F32, DEC_BF16 = _dec_cases()


@pytest.mark.parametrize("cfg", DEC_F32, ids=[c.name for c in DEC_F32])
def test_decoder_block_dropout_f32(cfg):
    from test_gpu_parity_decoder import _check
    _check(cfg, TOL_F32, TOL_F32, TOL_F32, TOL_F32)


@pytest.mark.parametrize("cfg", DEC_BF16, ids=[c.name for c in DEC_BF16])
def test_decoder_block_dropout_bf16(cfg):
    from test_gpu_parity_decoder import _check_bf16
    _check_bf16(cfg)


def _stack_cases():
    import test_gpu_parity_stack as TS
    f32 = [_drop_stack(TS.F32_CASES[0], name="drop_stack_f32"), _drop_stack(TS.F32_CASES[1], name="drop_stack_f32_tied"),
           _drop_stack(TS.F32_CASES[2], float(np.float32(0.25)), 3, name="drop_stack_f32_remat")]
    bf = [_drop_stack(TS.BF16_CASES[0], name="drop_stack_bf16"), _drop_stack(TS.BF16_CASES[1], name="drop_stack_bf16_tied"),
          _drop_stack(TS.BF16_CASES[5], name="drop_stack_bf16_ragged")]
    ef32 = [_drop_encdec(TS.EC_F32[0], name="drop_ec_f32"),
            _drop_encdec(TS.EC_F32[1], float(np.float32(0.2)), 21, 22, name="drop_ec_f32_tied_remat")]
    ebf = [_drop_encdec(TS.EC_BF16[0], name="drop_ec_bf16"), _drop_encdec(TS.EC_BF16[2], name="drop_ec_bf16_ragged")]
    return f32, bf, ef32, ebf


ST_F32, ST_BF16, EC_F32, EC_BF16 = _stack_cases()


@pytest.mark.parametrize("sc", ST_F32, ids=[c.name for c in ST_F32])
def test_stack_dropout_f32(sc):
    from test_gpu_parity_stack import _compare
    _compare(sc, 1e-5, TOL_F32[0])


@pytest.mark.parametrize("sc", ST_BF16, ids=[c.name for c in ST_BF16])
def test_stack_dropout_bf16(sc):
    from test_gpu_parity_stack import _compare
    _compare(sc, 5e-4 / (1.0 - RATE))


def test_stack_dropout_remat_replays_the_masks():
    """Recomputing a layer in the backward regenerates the same masks: gradients equal those of the stashed run
    (up to the order of the float32 atomic additions of the weight gradients)."""
    import test_gpu_parity_stack as TS
    sc = ST_BF16[0]
    w, tokens, targets = TS._case(sc)
    l1, g1 = TS._run(sc, w, tokens, targets)
    l2, g2 = TS._run(replace(sc, remat=True), w, tokens, targets)
    assert l1 == l2
    from parity_util import to_np
    for l in range(sc.n_layers):
        for name in g1["layers"][l]:
            a, b = to_np(g1["layers"][l][name]), to_np(g2["layers"][l][name])
            assert np.abs(a - b).max() <= 1e-4 * (np.abs(a).max() + 1e-30), (l, name)


@pytest.mark.parametrize("ec", EC_F32, ids=[c.name for c in EC_F32])
def test_encdec_dropout_f32(ec):
    from test_gpu_parity_stack import _ec_compare
    _ec_compare(ec, 1e-5, TOL_F32[0])


@pytest.mark.parametrize("ec", EC_BF16, ids=[c.name for c in EC_BF16])
def test_encdec_dropout_bf16(ec):
    from test_gpu_parity_stack import _ec_compare
    _ec_compare(ec, 5e-4 / (1.0 - RATE))
