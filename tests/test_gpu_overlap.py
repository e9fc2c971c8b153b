"""Weight-gradient GEMMs on the library's second stream: the results of every backward entry point equal
those of the single-stream run (dx and the loss bit for bit, weight gradients up to the order of the float32
atomic additions), also when calls follow each other without host synchronisation."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import synth_inputs as SI
from parity_util import make_case, make_decoder_case, to_dev, to_np, upload_case

pytestmark = pytest.mark.gpu


def _P():
    import paper_2203_17189_amd as P
    return P


@pytest.fixture
def overlap():
    P = _P()
    P.t5_wgrad_overlap_enable(True)
    try:
        yield P
    finally:
        torch.cuda.synchronize()
        P.t5_wgrad_overlap_enable(False)


def _close(a, b, what):
    a, b = to_np(a), to_np(b)
    assert np.abs(a - b).max() <= 1e-4 * (np.abs(a).max() + 1e-30), what


BLK = SI.BlockConfig("ovl_bf16", 90, batch=4, seq=256, d_model=256, n_heads=4, d_kv=64, d_ff=512, attn_scale=0.125)


def test_block_backward_overlapped_equals_serial(overlap):
    P = overlap
    w, x, dy = make_case(BLK)
    dw, tx, tdy = upload_case(BLK, w, x, dy)
    y, stash = P.t5_block_fwd(BLK, tx, dw)
    runs = [P.t5_block_bwd(BLK, tdy, tx, dw, stash) for _ in range(3)]     # back to back, no host sync in between
    torch.cuda.synchronize()
    P.t5_wgrad_overlap_enable(False)
    dx0, g0 = P.t5_block_bwd(BLK, tdy, tx, dw, stash)
    torch.cuda.synchronize()
    for dx, g in runs:
        assert torch.equal(dx, dx0)
        for k in g0:
            _close(g[k], g0[k], k)


def test_decoder_backward_overlapped_equals_serial(overlap):
    P = overlap
    cfg = replace(BLK, name="ovl_dec", index=91, causal=True, enc_seq=128)
    w, x, enc, dy = make_decoder_case(cfg)
    dw = {k: to_dev(v, cfg.dtype) for k, v in w.items()}
    tx, te, tdy = to_dev(x, cfg.dtype), to_dev(enc, cfg.dtype), to_dev(dy, cfg.dtype)
    y, stash = P.t5_decoder_block_fwd(cfg, tx, te, dw)
    dx1, de1, g1 = P.t5_decoder_block_bwd(cfg, tdy, tx, te, dw, stash)
    torch.cuda.synchronize()
    P.t5_wgrad_overlap_enable(False)
    dx0, de0, g0 = P.t5_decoder_block_bwd(cfg, tdy, tx, te, dw, stash)
    torch.cuda.synchronize()
    assert torch.equal(dx1, dx0) and torch.equal(de1, de0)
    for k in g0:
        _close(g1[k], g0[k], k)


@pytest.mark.parametrize("remat", [False, True])
def test_stack_overlapped_equals_serial(overlap, remat):
    import test_gpu_parity_stack as TS
    P = overlap
    sc = replace(TS.BF16_CASES[0], n_layers=3, remat=remat)
    w, tokens, targets = TS._case(sc)
    l1, g1 = TS._run(sc, w, tokens, targets)
    P.t5_wgrad_overlap_enable(False)
    l0, g0 = TS._run(sc, w, tokens, targets)
    assert l1 == l0
    for k in ("embedding", "rel_table", "final_scale", "logits_w"):
        _close(g1[k], g0[k], k)
    for l in range(sc.n_layers):
        for k in g0["layers"][l]:
            _close(g1["layers"][l][k], g0["layers"][l][k], (l, k))


def test_captured_pass_stays_on_the_callers_stream(overlap):
    """With the second stream enabled, a backward recorded into a graph runs on the capturing stream alone:
    the replays match the eager (overlapped) results."""
    P = overlap
    from paper_2203_17189_amd import binding as B
    w, x, dy = make_case(BLK)
    dw, tx, tdy = upload_case(BLK, w, x, dy)
    mk = lambda: dict(y=torch.empty_like(tx), dx=torch.empty_like(tx), grads=B.alloc_grads(BLK, dw),
                      stash=torch.empty(P.t5_block_stash_bytes(BLK), dtype=torch.uint8, device="cuda"),
                      ws=torch.empty(P.t5_block_workspace_bytes(BLK), dtype=torch.uint8, device="cuda"))
    eager, graph = mk(), mk()

    def step(b):
        P.t5_block_fwd(BLK, tx, dw, y=b["y"], stash=b["stash"], workspace=b["ws"])
        P.t5_block_bwd(BLK, tdy, tx, dw, b["stash"], dx=b["dx"], grads=b["grads"], workspace=b["ws"])

    step(graph)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(graph)
    for rep in range(3):
        graph["dx"].zero_()
        g.replay()
        step(eager)
        torch.cuda.synchronize()
        assert torch.equal(graph["dx"], eager["dx"]), rep
        for k in eager["grads"]:
            _close(graph["grads"][k], eager["grads"][k], (rep, k))


def test_encdec_overlapped_equals_serial(overlap):
    import test_gpu_parity_stack as TS
    P = overlap
    ec = TS.EC_BF16[0]
    w = SI.make_encdec_weights(ec)
    SI.make_encdec_random_scales(ec, w)
    enc_tokens, dec_tokens, targets = SI.make_encdec_tokens(ec, ignore_fraction=0.15)
    dw, te, td, tg = TS._ec_upload(ec, w, enc_tokens, dec_tokens, targets)
    l1, g1 = P.t5_encdec_loss_and_grad(ec, te, td, tg, dw)
    torch.cuda.synchronize()
    P.t5_wgrad_overlap_enable(False)
    l0, g0 = P.t5_encdec_loss_and_grad(ec, te, td, tg, dw)
    torch.cuda.synchronize()
    assert float(l1.item()) == float(l0.item())
    for k in [k for k in g0 if not k.endswith("_layers")]:
        _close(g1[k], g0[k], k)
    for side in ("enc_layers", "dec_layers"):
        for l in range(len(g0[side])):
            for k in g0[side][l]:
                _close(g1[side][l][k], g0[side][l][k], (side, l, k))
