"""End to end: a few training steps of a small stack -- loss and gradients from t5_stack_loss_and_grad,
then the Adafactor update of every tensor through adafactor_step_multi -- against the same steps taken
with the float64 oracle; and a longer bf16 run whose loss has to fall."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import synth_inputs as SI
from oracle import t5_oracle as O
from parity_util import to_np

pytestmark = pytest.mark.gpu

BLK = SI.BlockConfig("train_f32", 95, batch=2, seq=24, d_model=32, n_heads=2, d_kv=8, d_ff=48, dtype="f32", causal=True)
SC = SI.StackConfig("train_f32", BLK, n_layers=2, vocab=40, z_loss=1e-3)


def _flat(w, g):
    """[(name, weight, gradient)] over the nested structures, in a fixed order."""
    out = [(k, w[k], g[k]) for k in sorted(g) if k != "layers"]
    for l, gl in enumerate(g["layers"]):
        out += [(f"L{l}.{k}", w["layers"][l][k], gl[k]) for k in sorted(gl)]
    return out


def _factored(name, arr):
    return arr.ndim == 2 and "rel_table" not in name and "embedding" not in name


def test_three_training_steps_follow_the_oracle():
    import paper_2203_17189_amd as P
    from paper_2203_17189_amd import binding as B
    import test_gpu_parity_stack as TS
    w, tokens, targets = TS._case(SC)
    dw, ttok, ttgt = TS._upload(SC, w, tokens, targets)
    grads = B.alloc_stack_grads(SC, dw)
    # float32 model: the tensors the stack reads are the optimizer's parameters
    opt = []
    for name, wt, gt in _flat(dw, grads):
        rows, cols = (wt.shape[0], wt.shape[1]) if wt.dim() == 2 else (1, wt.numel())
        fact = wt.dim() == 2 and "rel_table" not in name and "embedding" not in name
        opt.append(dict(param=wt, grad=gt, factored=fact, v_row=torch.zeros(rows, device="cuda"),
                        v_col=torch.zeros(cols, device="cuda"), v_full=torch.zeros(rows, cols, device="cuda")))
    state = {}
    lr = 3e-2
    for step in (1, 2, 3):
        loss_ref, saved = O.stack_loss(SC, tokens, targets, w)
        g_ref = O.stack_loss_grad(SC, w, saved)
        loss_gpu, _ = P.t5_stack_loss_and_grad(SC, ttok, ttgt, dw, grads=grads)
        P.adafactor_step_multi(opt, step=step, lr=lr)
        torch.cuda.synchronize()
        assert abs(float(loss_gpu.item()) - loss_ref) <= 2e-5 * max(1.0, abs(loss_ref)), (step, float(loss_gpu.item()), loss_ref)
        for name, arr, grad in _flat(w, g_ref):
            p2 = arr.reshape(1, -1) if arr.ndim == 1 else arr
            g2 = grad.reshape(p2.shape)
            fact = _factored(name, arr)
            st = state.get(name) or O.adafactor_zero_state(p2.shape[0], p2.shape[1], fact)
            new, state[name] = O.adafactor_step(p2, g2, st, step=step, lr=lr, factored=fact)
            arr[...] = new.reshape(arr.shape)
    for (name, arr, _), (_, wt, _) in zip(_flat(w, g_ref), _flat(dw, grads)):
        err = np.abs(to_np(wt) - arr).max() / (np.sqrt(np.mean(arr * arr)) + 1e-30)
        assert err <= 2e-3, (name, err)    # three updates of size lr * RMS(W): float32 differences in U are amplified by lr only


def test_bf16_training_loss_falls():
    """bf16 model with float32 masters: 30 steps on one fixed batch bring the loss well below its start
    (ln V for random logits)."""
    import paper_2203_17189_amd as P
    from paper_2203_17189_amd import binding as B
    import test_gpu_parity_stack as TS
    sc = replace(TS.BF16_CASES[0], n_layers=2)
    w, tokens, targets = TS._case(sc)
    dw, ttok, ttgt = TS._upload(sc, w, tokens, targets)
    grads = B.alloc_stack_grads(sc, dw)
    opt = []
    for name, wt, gt in _flat(dw, grads):
        master = wt.float().contiguous()
        rows, cols = (master.shape[0], master.shape[1]) if master.dim() == 2 else (1, master.numel())
        fact = master.dim() == 2 and "rel_table" not in name and "embedding" not in name
        opt.append(dict(param=master, grad=gt, factored=fact, v_row=torch.zeros(rows, device="cuda"),
                        v_col=torch.zeros(cols, device="cuda"), v_full=torch.zeros(rows, cols, device="cuda"),
                        bf16_copy_out=wt))
    ws = torch.empty(P.t5_stack_workspace_bytes(sc), dtype=torch.uint8, device="cuda")
    losses = []
    for step in range(1, 31):
        loss, _ = P.t5_stack_loss_and_grad(sc, ttok, ttgt, dw, grads=grads, workspace=ws)
        P.adafactor_step_multi(opt, step=step, lr=1e-2)
        losses.append(float(loss.item()))
    print("loss", [round(v, 3) for v in losses[::5]], round(losses[-1], 3))
    assert np.isfinite(losses).all()
    assert losses[0] > 0.9 * np.log(sc.vocab)
    assert losses[-1] < 0.6 * losses[0], losses
