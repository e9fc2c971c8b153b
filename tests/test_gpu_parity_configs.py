"""GPU parity at the shapes of the five workload configurations.

Sequences are independent through the block, so the float64 oracle is run at a reduced batch b0
(full sequence length, widths, heads and d_ff) and the HIP path is called with the same batch so
that the weight-gradient sums match.  In addition, at the full batch of the configuration that
bench.py times, the first b0 sequences of y and dx are compared with the oracle (the batch only
adds independent rows), and properties that hold at any size are checked.

Tolerances (error e_i = |gpu_i - ref_i| / max(|ref_i|, RMS(ref)), max and mean per tensor): the stated
2e-2 / 2e-3 for every tensor whose ideal bf16-operand floor (tests/bf16_model.py, evaluated for the same
case) is at or under it, floor x 1.25 for the others (parity_util.tol_from_floor).  With attn_scale = 1
and unit-variance q, k the logits have standard deviation sqrt(d_kv); every bf16 rounding of n1, q and k is
multiplied by that factor inside the softmax, and the floor of that reading lies above the stated bound
for every tensor.
"""
from dataclasses import replace

import numpy as np
import pytest
import torch

import synth_inputs as SI
from oracle import t5_oracle as O
from parity_util import block_floors, check_bf16, make_case, rel_err, run_block_gpu, to_dev, to_np

pytestmark = pytest.mark.gpu

CASES = [("c2_small", 2), ("c3_base", 2), ("c4_gpt_causal", 1), ("c5_xl", 1), ("c7_xl_tp8_share", 1)]


def _scaled(cfg):
    return replace(cfg, attn_scale=cfg.d_kv ** -0.5)


@pytest.mark.parametrize("name,b0", CASES)
def test_config_reduced_batch_scaled_logits(name, b0):
    cfg = _scaled(SI.CONFIGS[name]).with_batch(b0)
    w, x, dy = make_case(cfg)
    y, saved = O.block_fwd(cfg, x, w)
    dx, g = O.block_bwd(cfg, dy, w, saved)
    gy, gdx, gg = run_block_gpu(cfg, w, x, dy)
    errs = {"y": rel_err(gy, y), "dx": rel_err(gdx, dx), **{k: rel_err(gg[k], g[k]) for k in g}}
    check_bf16(name + " scaled", errs, block_floors(cfg, w, x, dy, (y, dx, g)))
    # the bias-table gradient sums to zero over buckets for every head (softmax Jacobian rows sum to 0)
    assert np.abs(gg["rel_table"].sum(0)).max() <= 1e-3 * np.abs(gg["rel_table"]).max() * 32


@pytest.mark.parametrize("name,b0", [("c2_small", 2), ("c3_base", 2), ("c4_gpt_causal", 1), ("c5_xl", 1)])
def test_config_literal_unscaled_logits(name, b0):
    """attn_scale = 1 (no 1/sqrt(d_kv)) with unit-variance q, k: logits of std sqrt(d_kv)."""
    cfg = SI.CONFIGS[name].with_batch(b0)
    assert cfg.attn_scale == 1.0
    w, x, dy = make_case(cfg)
    y, saved = O.block_fwd(cfg, x, w)
    dx, g = O.block_bwd(cfg, dy, w, saved)
    gy, gdx, gg = run_block_gpu(cfg, w, x, dy)
    errs = {"y": rel_err(gy, y), "dx": rel_err(gdx, dx), **{k: rel_err(gg[k], g[k]) for k in g}}
    check_bf16(name + " literal", errs, block_floors(cfg, w, x, dy, (y, dx, g)))


@pytest.mark.parametrize("name,b0", [("c2_small", 2), ("c3_base", 1), ("c4_gpt_causal", 1), ("c5_xl", 1)])
def test_bench_workload_full_batch_sampled(name, b0):
    """A workload at its full batch, as bench.py launches it: the first b0 sequences against the oracle
    (sequences are independent through the block), run-to-run determinism of y and dx, finite gradients and
    the zero column sums of the bias-table gradient."""
    import paper_2203_17189_amd as P
    cfg = _scaled(SI.CONFIGS[name])
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
    # y and dx of a sequence do not depend on the other sequences: the floor of the sampled rows is the floor
    # of the same rows run alone
    check_bf16(name + " full batch sample", errs, block_floors(small, w, x[:b0], dy[:b0], (y, dx, g_small)),
               only=("y", "dx"))
    assert torch.equal(gy, gy2) and torch.equal(gdx, gdx2)          # y, dx use no atomics
    assert all(torch.isfinite(v).all() for v in gg.values())
    tab = to_np(gg["rel_table"])
    assert np.abs(tab.sum(0)).max() <= 1e-3 * np.abs(tab).max() * 32


def test_c3_adafactor_on_block_gradients():
    """Adafactor on the float32 gradients the block produced, against the oracle fed the same
    gradients (so only the optimizer arithmetic is compared), t = 1, 2."""
    import paper_2203_17189_amd as P
    cfg = _scaled(SI.CONFIGS["c3_base"]).with_batch(1)
    w, x, dy = make_case(cfg)
    dw = {k: to_dev(v, cfg.dtype) for k, v in w.items()}
    tx = to_dev(x, cfg.dtype)
    for name in ("wi0", "wo", "rel_table", "ln1_scale"):
        master = dw[name].float().contiguous()
        rows, cols = (master.shape[0], master.shape[1]) if master.dim() == 2 else (1, master.numel())
        fact = master.dim() == 2 and name != "rel_table"
        st = O.adafactor_zero_state(rows, cols, fact)
        vr, vc = torch.zeros(rows, device="cuda"), torch.zeros(cols, device="cuda")
        vf = torch.zeros(rows, cols, device="cuda")
        ref = to_np(master).reshape(rows, cols)
        for t in (1, 2):
            _, tdy = make_case(cfg, seed_offset=t)[1:]
            y_, stash = P.t5_block_fwd(cfg, tx, dw)
            _, gg = P.t5_block_bwd(cfg, to_dev(tdy, cfg.dtype), tx, dw, stash)
            torch.cuda.synchronize()
            gnp = to_np(gg[name]).reshape(rows, cols)
            ref, st = O.adafactor_step(ref, gnp, st, step=t, lr=1e-2, factored=fact)
            P.adafactor_step(master, gg[name], step=t, lr=1e-2, factored=fact, v_row=vr, v_col=vc, v_full=vf)
            torch.cuda.synchronize()
            e = rel_err(to_np(master), ref)
            assert e[0] <= 2e-5, (name, t, e)
