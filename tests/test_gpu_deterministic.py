"""The reproducible mode (t5_block_cfg.deterministic): weight gradients and the bias-table gradient come out
bit-identical from run to run -- their partial sums are added in a fixed order by a second pass instead of
meeting in float32 atomics -- and agree with the default mode to float32 rounding."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import synth_inputs as SI
from parity_util import make_case, make_decoder_case, to_dev, to_np

pytestmark = pytest.mark.gpu


def _run_block(P, cfg, dw, tx, tdy, accumulate_into=None):
    y, stash = P.t5_block_fwd(cfg, tx, dw)
    if accumulate_into is None:
        dx, g = P.t5_block_bwd(cfg, tdy, tx, dw, stash)
    else:
        dx, g = P.t5_block_bwd(cfg, tdy, tx, dw, stash, grads=accumulate_into, accumulate=True)
    torch.cuda.synchronize()
    return y, dx, g


@pytest.mark.parametrize("name,batch", [("c2_small", 64), ("c3_base", 16), ("c4_gpt_causal", 2)])
def test_block_gradients_bit_reproducible(name, batch):
    import paper_2203_17189_amd as P
    base = SI.CONFIGS[name].with_batch(batch)
    cfg = replace(base, deterministic=True)
    assert P.t5_block_workspace_bytes(cfg) > P.t5_block_workspace_bytes(base)    # room for the partial sums
    w, x, dy = make_case(cfg)
    dw = {k: to_dev(v, cfg.dtype) for k, v in w.items()}
    tx, tdy = to_dev(x, cfg.dtype), to_dev(dy, cfg.dtype)
    y1, dx1, g1 = _run_block(P, cfg, dw, tx, tdy)
    # other work in between, so that the second run meets a different machine state
    _run_block(P, base, dw, tx, tdy)
    y2, dx2, g2 = _run_block(P, cfg, dw, tx, tdy)
    assert torch.equal(y1, y2) and torch.equal(dx1, dx2)
    for k in g1:
        assert torch.equal(g1[k], g2[k]), k
    # same numbers as the default mode, up to the order of float32 additions
    _, dx0, g0 = _run_block(P, base, dw, tx, tdy)
    assert torch.equal(dx0, dx1)
    for k in g1:
        a, b = to_np(g0[k]), to_np(g1[k])
        assert np.abs(a - b).max() <= 2e-5 * np.abs(a).max() + 1e-12, k
    # accumulate: a second backward adds onto the first, again bit-reproducibly
    acc1 = {k: v.clone() for k, v in g1.items()}
    acc2 = {k: v.clone() for k, v in g1.items()}
    _run_block(P, cfg, dw, tx, tdy, accumulate_into=acc1)
    _run_block(P, cfg, dw, tx, tdy, accumulate_into=acc2)
    for k in g1:
        assert torch.equal(acc1[k], acc2[k]), k
        a = to_np(g1[k])
        assert np.abs(to_np(acc1[k]) - 2 * a).max() <= 4e-5 * np.abs(a).max() + 1e-12, k


def test_decoder_layer_gradients_bit_reproducible():
    import paper_2203_17189_amd as P
    cfg = replace(SI.CONFIGS["c6_dec_base"].with_batch(16), deterministic=True)
    w, x, enc, dy = make_decoder_case(cfg)
    dw = {k: to_dev(v, cfg.dtype) for k, v in w.items()}
    tx, te, tdy = to_dev(x, cfg.dtype), to_dev(enc, cfg.dtype), to_dev(dy, cfg.dtype)
    outs = []
    for _ in range(2):
        y, stash = P.t5_decoder_block_fwd(cfg, tx, te, dw)
        dx, denc, g = P.t5_decoder_block_bwd(cfg, tdy, tx, te, dw, stash)
        torch.cuda.synchronize()
        outs.append((dx, denc, g))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    for k in outs[0][2]:
        assert torch.equal(outs[0][2][k], outs[1][2][k]), k


@pytest.mark.parametrize("tied", [False, True], ids=["untied", "tied"])
def test_stack_gradients_bit_reproducible(tied):
    """A stack in the reproducible mode: every gradient -- the layers' weights, the shared bias table, the final
    norm's scale, the output matrix (k-slices of its GEMM summed in a fixed order, chunk after chunk) and the
    embedding (one wave per vocabulary row adds the rows of its tokens in position order; with tied logits on top
    of the output-matrix term) -- is bit-identical between two runs, and agrees with the default mode."""
    import paper_2203_17189_amd as P
    import test_gpu_parity_stack as TS
    blk = replace(TS.BF_BLK, index=58, batch=16, seq=256, deterministic=True)
    sc = SI.StackConfig("stack_det", blk, n_layers=3, vocab=512, tied_logits=tied)
    w, tokens, targets = TS._case(sc)
    l1, g1 = TS._run(sc, w, tokens, targets)
    l2, g2 = TS._run(sc, w, tokens, targets)
    assert l1 == l2
    top = [k for k in g1 if k != "layers"]
    assert "embedding" in top and ("logits_w" in top) == (not tied), top
    for k in top:
        assert torch.equal(g1[k], g2[k]), k
    for l in range(sc.n_layers):
        for n in g1["layers"][l]:
            assert torch.equal(g1["layers"][l][n], g2["layers"][l][n]), (l, n)
    # same sums as the default mode, in another order
    sd = SI.StackConfig("stack_det", replace(blk, deterministic=False), n_layers=3, vocab=512, tied_logits=tied)
    _, g0 = TS._run(sd, w, tokens, targets)
    for k in top:
        a, b = g1[k].float(), g0[k].float()
        assert (a - b).abs().max().item() <= 2e-5 * (b.abs().max().item() + 1e-30), k


def test_encdec_gradients_bit_reproducible():
    """The encoder-decoder pair in the reproducible mode: both token streams add into one embedding gradient (the
    decoder's first, then the encoder's, each in position order), and every gradient is bit-identical between runs."""
    import paper_2203_17189_amd as P
    import test_gpu_parity_stack as TS
    ec = SI._encdec("ec_det", 79, 2, 256, 128, 128, 2, 64, 256, 2, 2, 512,
                    block=dict(attn_scale=64 ** -0.5, deterministic=True))
    w = SI.make_encdec_weights(ec)
    enc_tokens, dec_tokens, targets = SI.make_encdec_tokens(ec, ignore_fraction=0.15)
    dw, te, td, tg = TS._ec_upload(ec, w, enc_tokens, dec_tokens, targets)
    outs = []
    for _ in range(2):
        loss, g = P.t5_encdec_loss_and_grad(ec, te, td, tg, dw)
        torch.cuda.synchronize()
        outs.append((float(loss.item()), g))
    assert outs[0][0] == outs[1][0]
    g1, g2 = outs[0][1], outs[1][1]
    for k in g1:
        if k.endswith("_layers"):
            for l in range(len(g1[k])):
                for n in g1[k][l]:
                    assert torch.equal(g1[k][l][n], g2[k][l][n]), (k, l, n)
        else:
            assert torch.equal(g1[k], g2[k]), k
