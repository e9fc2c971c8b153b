"""GPU parity of dropout: the keep masks bit for bit against the oracle's generator, and the block's
forward and backward with dropout at its four sites against the float64 oracle."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import synth_inputs as SI
from oracle import t5_oracle as O
from parity_util import (TOL_BF16_ACT, TOL_BF16_DW, TOL_BF16_DX, TOL_F32, drop_tol, make_case, rel_err, relu_aware,
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
    ey, edx = rel_err(gy, y), rel_err(gdx, dx)
    print(cfg.name, "y", ey, "dx", edx, {k: rel_err(gg[k], g[k]) for k in g})
    p = cfg.dropout_rate
    tol_y = drop_tol(TOL_BF16_ACT, p, False)
    assert ey[0] <= tol_y[0] and ey[1] <= tol_y[1], ey
    tol_dx, tol_dw = relu_aware(cfg, drop_tol(TOL_BF16_DX, p, True)), relu_aware(cfg, drop_tol(TOL_BF16_DW, p, True))
    assert edx[0] <= tol_dx[0] and edx[1] <= tol_dx[1], edx
    for name in g:
        e = rel_err(gg[name], g[name])
        tol = drop_tol(TOL_BF16_DW, p, True) if name == "wo_ff" else tol_dw
        assert e[0] <= tol[0] and e[1] <= tol[1], (name, e)


# ------------------------------------------------------------------ workload shapes (matrix-unit kernels)
def _named(name, b):
    cfg = SI.CONFIGS[name]
    return replace(cfg, attn_scale=cfg.d_kv ** -0.5, dropout_rate=RATE, dropout_seed=SEED + 5).with_batch(b)


@pytest.mark.parametrize("name,b0", [("c3_base", 2), ("c4_gpt_causal", 1)])
def test_config_dropout_reduced_batch(name, b0):
    """Full sequence length, widths and heads of a workload at a reduced batch (sequences are independent
    through the block): several query and key tiles per head in the fused attention kernels."""
    from parity_util import TOL_BF16_DW_NAMED, TOL_BF16_DX_NAMED
    cfg = _named(name, b0)
    w, x, dy = make_case(cfg)
    y, saved = O.block_fwd(cfg, x, w)
    dx, g = O.block_bwd(cfg, dy, w, saved)
    gy, gdx, gg = run_block_gpu(cfg, w, x, dy)
    ey, edx = rel_err(gy, y), rel_err(gdx, dx)
    print(name, "y", ey, "dx", edx, {k: tuple(round(v, 5) for v in rel_err(gg[k], g[k])) for k in g})
    tol_y, tol_dx = drop_tol(TOL_BF16_ACT, RATE, False), drop_tol(TOL_BF16_DX_NAMED, RATE, True)
    tol_dw = drop_tol(TOL_BF16_DW_NAMED, RATE, True)
    assert ey[0] <= tol_y[0] and ey[1] <= tol_y[1], ("y", ey)
    assert edx[0] <= tol_dx[0] and edx[1] <= tol_dx[1], ("dx", edx)
    for k in g:
        e = rel_err(gg[k], g[k])
        assert e[0] <= tol_dw[0] and e[1] <= tol_dw[1], (k, e)


def test_dropout_full_batch_sampled():
    """c2_small at its full batch with dropout, as bench.py --dropout launches it: the first 2 sequences of y
    and dx against the oracle (the masks of a sequence depend on its own batch index only), and
    run-to-run determinism."""
    from parity_util import TOL_BF16_DX_NAMED, to_dev, to_np
    P = _P()
    cfg = _named("c2_small", SI.CONFIGS["c2_small"].batch)
    b0 = 2
    w = SI.make_weights(cfg)
    x, dy = SI.make_activations(cfg)
    small = cfg.with_batch(b0)
    y, saved = O.block_fwd(small, x[:b0], w)
    dx, _ = O.block_bwd(small, dy[:b0], w, saved)
    dw = {k: to_dev(v, cfg.dtype) for k, v in w.items()}
    tx, tdy = to_dev(x, cfg.dtype), to_dev(dy, cfg.dtype)
    gy, stash = P.t5_block_fwd(cfg, tx, dw)
    gdx, gg = P.t5_block_bwd(cfg, tdy, tx, dw, stash)
    gy2, stash2 = P.t5_block_fwd(cfg, tx, dw)
    gdx2, _ = P.t5_block_bwd(cfg, tdy, tx, dw, stash2)
    torch.cuda.synchronize()
    ey, edx = rel_err(to_np(gy[:b0]), y), rel_err(to_np(gdx[:b0]), dx)
    print("full batch sample with dropout: y", ey, "dx", edx)
    tol_y, tol_dx = drop_tol(TOL_BF16_ACT, RATE, False), drop_tol(TOL_BF16_DX_NAMED, RATE, True)
    assert ey[0] <= tol_y[0] and ey[1] <= tol_y[1], ey
    assert edx[0] <= tol_dx[0] and edx[1] <= tol_dx[1], edx
    assert torch.equal(gy, gy2) and torch.equal(gdx, gdx2)
    assert all(torch.isfinite(v).all() for v in gg.values())
