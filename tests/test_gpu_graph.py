"""The entry points allocate nothing, synchronise nothing and enqueue only kernels on the caller's stream,
so a caller can record them into a HIP graph.  Each test captures a step, replays it several times with
other (eager) work and synchronisations in between, and checks every replay against the eager result on
the same inputs."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import synth_inputs as SI
from parity_util import make_case, to_dev, to_np

pytestmark = pytest.mark.gpu


def test_block_step_in_a_graph_matches_eager():
    import paper_2203_17189_amd as P
    from paper_2203_17189_amd import binding as B
    cfg = SI.BlockConfig("graph_blk", 90, batch=2, seq=256, d_model=128, n_heads=2, d_kv=64, d_ff=256, causal=True,
                         attn_scale=64 ** -0.5)
    w, x, dy = make_case(cfg)
    dw = {k: to_dev(v, cfg.dtype) for k, v in w.items()}
    tx, tdy = to_dev(x, cfg.dtype), to_dev(dy, cfg.dtype)
    mk = lambda: dict(y=torch.empty_like(tx), dx=torch.empty_like(tx), grads=B.alloc_grads(cfg, dw),
                      stash=torch.empty(P.t5_block_stash_bytes(cfg), dtype=torch.uint8, device="cuda"),
                      ws=torch.empty(P.t5_block_workspace_bytes(cfg), dtype=torch.uint8, device="cuda"))
    eager, graph = mk(), mk()

    def step(b):
        P.t5_block_fwd(cfg, tx, dw, y=b["y"], stash=b["stash"], workspace=b["ws"])
        P.t5_block_bwd(cfg, tdy, tx, dw, b["stash"], dx=b["dx"], grads=b["grads"], workspace=b["ws"])

    step(graph)                      # first launches outside the capture (kernel attributes are set there)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(graph)
    for rep in range(4):
        _, x2, dy2 = make_case(cfg, seed_offset=rep + 1)
        tx.copy_(to_dev(x2, cfg.dtype)); tdy.copy_(to_dev(dy2, cfg.dtype))
        graph["y"].zero_(); graph["dx"].zero_()
        g.replay()
        step(eager)                  # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(graph["y"], eager["y"]) and torch.equal(graph["dx"], eager["dx"]), rep
        for k in eager["grads"]:
            a = to_np(eager["grads"][k])
            assert np.abs(to_np(graph["grads"][k]) - a).max() <= 1e-4 * (np.abs(a).max() + 1e-30), (rep, k)


@pytest.mark.parametrize("remat", [True, False])
def test_stack_step_in_a_graph_matches_eager(remat):
    # remat: per-layer weight-gradient launches; without it the grouped launches, whose pointer tables are
    # written by kernels inside the captured step
    import paper_2203_17189_amd as P
    from paper_2203_17189_amd import binding as B
    blk = SI.BlockConfig("graph_stack", 91, batch=2, seq=128, d_model=128, n_heads=2, d_kv=64, d_ff=256, causal=True,
                         attn_scale=64 ** -0.5)
    sc = SI.StackConfig("graph_stack", blk, n_layers=2, vocab=512, remat=remat)
    w = SI.make_stack_weights(sc)
    dw = {k: to_dev(v, blk.dtype) for k, v in w.items() if k != "layers"}
    dw["layers"] = [{k: to_dev(v, blk.dtype) for k, v in lw.items()} for lw in w["layers"]]
    tok, tgt = SI.make_tokens(sc)
    ttok, ttgt = torch.from_numpy(tok).cuda(), torch.from_numpy(tgt).cuda()
    mk = lambda: dict(grads=B.alloc_stack_grads(sc, dw), loss=torch.zeros(1, device="cuda"),
                      ws=torch.empty(P.t5_stack_workspace_bytes(sc), dtype=torch.uint8, device="cuda"))
    eager, graph = mk(), mk()
    step = lambda b: P.t5_stack_loss_and_grad(sc, ttok, ttgt, dw, grads=b["grads"], workspace=b["ws"], loss=b["loss"])
    step(graph)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(graph)
    for rep in range(3):
        tok2, tgt2 = SI.make_tokens(sc, seed_offset=rep + 1)
        ttok.copy_(torch.from_numpy(tok2).cuda()); ttgt.copy_(torch.from_numpy(tgt2).cuda())
        graph["loss"].zero_()
        g.replay()
        step(eager)
        torch.cuda.synchronize()
        assert torch.equal(graph["loss"], eager["loss"]), rep
        for k in ("embedding", "rel_table", "final_scale", "logits_w"):
            a = to_np(eager["grads"][k])
            assert np.abs(to_np(graph["grads"][k]) - a).max() <= 1e-4 * (np.abs(a).max() + 1e-30), (rep, k)
        for l in range(sc.n_layers):
            for k, v in eager["grads"]["layers"][l].items():
                a = to_np(v)
                assert np.abs(to_np(graph["grads"]["layers"][l][k]) - a).max() <= 1e-4 * (np.abs(a).max() + 1e-30), (rep, l, k)
