#!/usr/bin/env python3
"""Benchmark of the T5.1.1 block hot path (forward + backward [+ Adafactor]) on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5_xl|c2_small|c3_base|c4_gpt_causal|c6_dec_base|c7_xl_tp8_share|s1_lm_base|e1_t5_base]

Prints ONE JSON line.  A "step" is one pass of the whole hot path over one batch of seeded
synthetic input already resident in HBM: t5_block_fwd + t5_block_bwd (t5_decoder_block_fwd/bwd for the
workload with cross-attention), plus adafactor_step_multi over the block weights for the workloads that
include the optimizer.  `value` is tokens/s of that step.
`roofline` describes the step's dominant kernel, timed with HIP events on the launch stream in a
second, instrumented pass over the same work; `cpu_baseline` is the float64 oracle timed on the host
cores on a bounded sample (fewer sequences, same shapes).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth_inputs as SI  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def gemm_step_flops(cfg) -> dict:
    """Algorithmic FLOPs of one launch of each MFMA step (2*M*N*K; attention counts the causal half)."""
    T, d, I, F, S = cfg.tokens, cfg.d_model, cfg.inner, cfg.d_ff, cfg.seq
    attn_f = 4.0 * T * S * I * (0.5 if cfg.causal else 1.0)
    Te, xattn_f = cfg.batch * cfg.enc_seq, 4.0 * T * cfg.enc_seq * I
    cross = {
        "gemm_xq": 2.0 * T * d * I, "gemm_xkv": 2.0 * Te * d * 2 * I, "xattn_fwd": xattn_f, "gemm_xo": 2.0 * T * I * d,
        "gemm_dxo": 2.0 * T * I * d, "gemm_dcx": 2.0 * T * I * d, "xattn_bwd_dq": xattn_f, "xattn_bwd_dkv": xattn_f,
        "gemm_dxq": 2.0 * T * d * I, "gemm_dxkv": 2.0 * Te * d * 2 * I, "gemm_denc": 2.0 * Te * d * 2 * I,
        "gemm_dnx": 2.0 * T * d * I,
    } if cfg.enc_seq > 0 else {}
    return {
        **cross,
        "gemm_qkv": 2.0 * T * d * 3 * I, "gemm_o": 2.0 * T * I * d, "gemm_wi_geglu": 2.0 * T * d * 2 * F,
        "gemm_wo": 2.0 * T * F * d, "attn_fwd": attn_f,
        "gemm_dwo_ff": 2.0 * T * F * d, "gemm_da_geglu_bwd": 2.0 * T * F * d, "gemm_dwi": 2.0 * T * d * 2 * F,
        "gemm_dn2": 2.0 * T * d * 2 * F, "gemm_dwo": 2.0 * T * I * d, "gemm_dc": 2.0 * T * I * d,
        # attention backward is two kernels; its model FLOPs (4 matmuls) are split evenly: the dq kernel
        # owns dP and dQ, the dk/dv kernel owns dV and dK (the recomputed scores are overhead, not work)
        "attn_bwd_dq": attn_f, "attn_bwd_dkv": attn_f, "gemm_dwqkv": 2.0 * T * d * 3 * I, "gemm_dn1": 2.0 * T * d * 3 * I,
    }


def cpu_baseline_stack(sc, sample_batch: int) -> dict:
    from oracle import t5_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    c = sc.with_batch(sample_batch)
    w = SI.make_stack_weights(c)
    tokens, targets = SI.make_tokens(c)
    t0 = time.perf_counter()
    loss, saved = O.stack_loss(c, tokens, targets, w)
    O.stack_loss_grad(c, w, saved)
    dt = time.perf_counter() - t0
    return {"value": c.block.tokens / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{sc.name} at batch {sample_batch} of {sc.block.batch} (same depth/seq/width/vocab), float64 "
                      f"numpy, {dt:.2f} s for one loss + gradient"}


def cpu_baseline_encdec(ec, sample_batch: int) -> dict:
    from oracle import t5_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    c = ec.with_batch(sample_batch)
    w = SI.make_encdec_weights(c)
    et, dtk, tg = SI.make_encdec_tokens(c)
    t0 = time.perf_counter()
    loss, saved = O.encdec_loss(c, et, dtk, tg, w)
    O.encdec_loss_grad(c, w, saved)
    dt = time.perf_counter() - t0
    return {"value": (c.enc_block.tokens + c.dec_block.tokens) / dt, "unit": "tokens/s", "cores": int(threads),
            "kind": "oracle",
            "sample": f"{ec.name} at batch {sample_batch} of {ec.dec_block.batch} (same depth/lengths/width/vocab), "
                      f"float64 numpy, {dt:.2f} s for one loss + gradient"}


def cpu_baseline(cfg, sample_batch: int) -> dict:
    from oracle import t5_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    c = cfg.with_batch(sample_batch)
    w = SI.make_weights(c)
    x, dy = SI.make_activations(c)
    enc = SI.make_encoder_output(c) if c.enc_seq > 0 else None
    t0 = time.perf_counter()
    if enc is None:
        y, saved = O.block_fwd(c, x, w)
        dx, g = O.block_bwd(c, dy, w, saved)
    else:
        y, saved = O.decoder_block_fwd(c, x, enc, w)
        dx, denc, g = O.decoder_block_bwd(c, dy, w, saved)
    if cfg.adafactor:
        for name, grad in g.items():
            p2 = w[name].reshape(-1, w[name].shape[-1]) if w[name].ndim > 1 else w[name].reshape(1, -1)
            g2 = grad.reshape(p2.shape)
            fact = min(p2.shape) >= 2 and name not in ("rel_table",)
            O.adafactor_step(p2, g2, O.adafactor_zero_state(p2.shape[0], p2.shape[1], fact), step=1, lr=1e-2,
                             factored=fact)
    dt = time.perf_counter() - t0
    return {"value": c.tokens / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{cfg.name} at batch {sample_batch} of {cfg.batch} (same seq/width), float64 numpy, "
                      f"{dt:.2f} s for one fwd+bwd" + ("+adafactor" if cfg.adafactor else "")}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c5_xl", choices=[k for k in SI.CONFIGS if k != "c1_tiny_f32"] + list(SI.STACK_CONFIGS) + list(SI.ENCDEC_CONFIGS))
    ap.add_argument("--cpu-sample-batch", type=int, default=0, help="0 = pick about 10-30 s of oracle work")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="record one step into a HIP graph after the warm-up and time K replays of it")
    ap.add_argument("--optimizer", action="store_true",
                    help="stack workloads: add the Adafactor update of every tensor of the model to the step")
    ap.add_argument("--overlap", action="store_true",
                    help="run the weight-gradient GEMMs of the backward on the library's second stream")
    ap.add_argument("--dropout", type=float, default=0.0,
                    help="dropout rate at every site of the workload (0 = the paper's pre-training recipe)")
    ap.add_argument("--deterministic", action="store_true",
                    help="weight and bias-table gradients summed in a fixed order (bit-reproducible backward)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run three 1 GiB device-to-device copies (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    import paper_2203_17189_amd as P
    from paper_2203_17189_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    sc = SI.STACK_CONFIGS.get(args.workload)
    ec = SI.ENCDEC_CONFIGS.get(args.workload)
    cfg = sc.block if sc is not None else (ec.dec_block if ec is not None else SI.CONFIGS[args.workload])
    if args.dropout > 0.0:
        import dataclasses
        drop = lambda c: dataclasses.replace(c, dropout_rate=float(np.float32(args.dropout)), dropout_seed=0x5EED5EED5EED)
        if sc is not None:
            sc = dataclasses.replace(sc, block=drop(sc.block))
        if ec is not None:
            ec = dataclasses.replace(ec, enc_block=drop(ec.enc_block), dec_block=drop(ec.dec_block))
        cfg = sc.block if sc is not None else (ec.dec_block if ec is not None else drop(cfg))
    if args.deterministic:
        import dataclasses
        det = lambda c: dataclasses.replace(c, deterministic=True)
        if sc is not None:
            sc = dataclasses.replace(sc, block=det(sc.block))
        if ec is not None:
            ec = dataclasses.replace(ec, enc_block=det(ec.enc_block), dec_block=det(ec.dec_block))
        cfg = sc.block if sc is not None else (ec.dec_block if ec is not None else det(cfg))
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).zero_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": 1 << 30, "copies": 3}))
        return 0

    # ---- seeded synthetic inputs, generated on the host, resident in HBM before timing
    dt_t = torch.bfloat16
    up = lambda v: torch.from_numpy(v.astype(np.float32)).to(dev).to(dt_t)
    if ec is not None:
        ws_host = SI.make_encdec_weights(ec)
        sw = {k: up(v) for k, v in ws_host.items() if not k.endswith("_layers")}
        for side in ("enc_layers", "dec_layers"):
            sw[side] = [{k: up(v) for k, v in lw.items()} for lw in ws_host[side]]
        del ws_host
        et_h, dt_h, tg_h = SI.make_encdec_tokens(ec)
        e_tok, s_tok, s_tgt = (torch.from_numpy(a).to(dev) for a in (et_h, dt_h, tg_h))
        s_grads = B.alloc_encdec_grads(ec, sw)
        s_ws = torch.empty(P.t5_encdec_workspace_bytes(ec), dtype=torch.uint8, device=dev)
        s_loss = torch.zeros(1, dtype=torch.float32, device=dev)
        w_host = {"rel_table": np.zeros((cfg.num_buckets, cfg.n_heads))}
    elif sc is not None:
        ws_host = SI.make_stack_weights(sc)
        sw = {k: up(v) for k, v in ws_host.items() if k != "layers"}
        sw["layers"] = [{k: up(v) for k, v in lw.items()} for lw in ws_host["layers"]]
        del ws_host
        tok_h, tgt_h = SI.make_tokens(sc)
        s_tok, s_tgt = torch.from_numpy(tok_h).to(dev), torch.from_numpy(tgt_h).to(dev)
        s_grads = B.alloc_stack_grads(sc, sw)
        s_ws = torch.empty(P.t5_stack_workspace_bytes(sc), dtype=torch.uint8, device=dev)
        s_loss = torch.zeros(1, dtype=torch.float32, device=dev)
        w_host = {"rel_table": np.zeros((cfg.num_buckets, cfg.n_heads))}
    else:
        w_host = SI.make_weights(cfg)
    w = {k: up(v) for k, v in w_host.items()}
    decoder = cfg.enc_seq > 0
    opt = None
    if sc is None and ec is None:
        # the seeded draws the parity tests use (float64 on the host, rounded once to bf16)
        x_h, dy_h = SI.make_activations(cfg)
        x, dy = up(x_h), up(dy_h)
        del x_h, dy_h
        y = torch.empty_like(x)
        dx = torch.empty_like(x)
        decoder = cfg.enc_seq > 0
        if decoder:
            enc = up(SI.make_encoder_output(cfg))
            denc = torch.empty_like(enc)
            stash = torch.empty(P.t5_decoder_block_stash_bytes(cfg), dtype=torch.uint8, device=dev)
            ws = torch.empty(P.t5_decoder_block_workspace_bytes(cfg), dtype=torch.uint8, device=dev)
            grads = B.alloc_decoder_grads(cfg, w)
        else:
            stash = torch.empty(P.t5_block_stash_bytes(cfg), dtype=torch.uint8, device=dev)
            ws = torch.empty(P.t5_block_workspace_bytes(cfg), dtype=torch.uint8, device=dev)
            grads = B.alloc_grads(cfg, w)
        opt = None
        if cfg.adafactor:
            opt = {}
            for name in grads:
                master = w[name].float().contiguous()
                rows, cols = (master.shape[0], master.shape[1]) if master.dim() == 2 else (1, master.numel())
                fact = master.dim() == 2 and name != "rel_table"
                opt[name] = dict(master=master, fact=fact,
                                 vr=torch.zeros(rows, device=dev), vc=torch.zeros(cols, device=dev),
                                 vf=None if fact else torch.zeros(rows, cols, device=dev))
            opt_tensors = [dict(param=o["master"], grad=grads[name], factored=o["fact"], v_row=o["vr"], v_col=o["vc"],
                                v_full=o["vf"], bf16_copy_out=w[name]) for name, o in opt.items()]
            opt_ws = torch.empty(max(P.adafactor_multi_workspace_bytes(opt_tensors), 256), dtype=torch.uint8, device=dev)

    def all_tensors(wt, gt, path=""):
        """(name, weight, gradient) of every tensor of a nested weight / gradient structure."""
        if isinstance(wt, dict):
            return [t for k in gt for t in all_tensors(wt[k], gt[k], f"{path}.{k}")]
        if isinstance(wt, list):
            return [t for i in range(len(gt)) for t in all_tensors(wt[i], gt[i], f"{path}[{i}]")]
        return [(path, wt, gt)]

    model_opt = None
    if args.optimizer and (sc is not None or ec is not None):
        # float32 master copies and second-moment state for every tensor; the bf16 weights the model reads are
        # refreshed by the update itself.  Matrices are factored, except the embedding and the bias tables.
        model_opt = []
        for name, wt, gt in all_tensors(sw, s_grads):
            master = wt.float().contiguous()
            rows, cols = (master.shape[0], master.shape[1]) if master.dim() == 2 else (1, master.numel())
            fact = master.dim() == 2 and "rel_table" not in name and "embedding" not in name
            model_opt.append(dict(param=master, grad=gt, factored=fact,
                                  v_row=torch.zeros(rows, device=dev) if fact else None,
                                  v_col=torch.zeros(cols, device=dev) if fact else None,
                                  v_full=None if fact else torch.zeros(rows, cols, device=dev), bf16_copy_out=wt))
        model_opt_ws = torch.empty(max(P.adafactor_multi_workspace_bytes(model_opt), 256), dtype=torch.uint8, device=dev)

    step_no = [0]

    def step():
        if ec is not None or sc is not None:
            if ec is not None:
                P.t5_encdec_loss_and_grad(ec, e_tok, s_tok, s_tgt, sw, grads=s_grads, workspace=s_ws, loss=s_loss)
            else:
                P.t5_stack_loss_and_grad(sc, s_tok, s_tgt, sw, grads=s_grads, workspace=s_ws, loss=s_loss)
            if model_opt is not None:
                step_no[0] += 1
                P.adafactor_step_multi(model_opt, step=step_no[0], lr=1e-3, workspace=model_opt_ws)
            return
        if decoder:
            P.t5_decoder_block_fwd(cfg, x, enc, w, y=y, stash=stash, workspace=ws)
            P.t5_decoder_block_bwd(cfg, dy, x, enc, w, stash, dx=dx, denc=denc, grads=grads, workspace=ws)
        else:
            P.t5_block_fwd(cfg, x, w, y=y, stash=stash, workspace=ws)
            P.t5_block_bwd(cfg, dy, x, w, stash, dx=dx, grads=grads, workspace=ws)
        if opt is not None:
            step_no[0] += 1
            P.adafactor_step_multi(opt_tensors, step=step_no[0], lr=1e-2, workspace=opt_ws)

    if args.overlap:
        P.t5_wgrad_overlap_enable(True)
    for _ in range(max(args.warmup, 1 if args.graph else 0)):
        step()
    torch.cuda.synchronize()
    run_step = step
    if args.graph:
        # the entry points only enqueue kernels on the current stream, so a step records as it is; the
        # Adafactor step number is frozen in the recording (it enters the kernels by value)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run_step = graph.replay
        run_step()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    step_tokens = cfg.tokens + (ec.enc_block.tokens if ec is not None else 0)
    tokens_per_s = step_tokens * args.steps / dt
    total_model_flops = sc.model_flops() if sc is not None else (ec.model_flops() if ec is not None else cfg.model_flops())
    model_tflops = total_model_flops / (ms_per_step * 1e-3) / 1e12

    # ---- instrumented pass: per-step HIP-event timing on the launch stream
    P.t5_step_timing_enable(True)
    n_prof = max(3, min(args.steps, 10))
    for _ in range(n_prof):
        step()
    torch.cuda.synchronize()
    timing = P.t5_step_timing_read()
    P.t5_step_timing_enable(False)
    flops = gemm_step_flops(cfg)
    if sc is not None or ec is not None:
        chunk = min(cfg.tokens, 16384)
        for name in ("gemm_logits", "gemm_dnf", "gemm_dlogits_w"):
            flops[name] = 2.0 * chunk * cfg.d_model * (sc or ec).vocab
    if ec is not None:
        # encoder and decoder layers launch the same step names at different token counts: per-step rates
        # would mix the two, so only the steps that exist on one side keep a FLOP count
        flops = {k: v for k, v in flops.items() if k.startswith(("gemm_x", "xattn", "gemm_dx", "gemm_dcx", "gemm_denc",
                                                                 "gemm_dnx", "gemm_logits", "gemm_dnf", "gemm_dlogits"))}
    per_kernel = {k: {"avg_ms": v[0] / v[1], "launches_per_step": v[1] / n_prof} for k, v in timing.items()}
    # a stack launches the weight-gradient GEMMs of all its layers together: one launch does n_layers problems
    n_lay = sc.n_layers if sc is not None else (ec.n_dec_layers if ec is not None else 1)
    for k in ("gemm_dwo_ff", "gemm_dwi", "gemm_dwo", "gemm_dwqkv", "gemm_dxo", "gemm_dxq", "gemm_dxkv"):
        if k in flops and k in per_kernel and n_lay > 1 and per_kernel[k]["launches_per_step"] < n_lay:
            flops[k] *= n_lay / per_kernel[k]["launches_per_step"]
    step_ms = {k: v["avg_ms"] * v["launches_per_step"] for k, v in per_kernel.items()}
    fwd_names = {"relpos_diag", "rmsnorm_fwd", "pack_weights", "gemm_qkv", "attn_fwd", "gemm_o", "gemm_wi_geglu",
                 "gemm_wi", "geglu_fwd", "gemm_wo", "gemm_xq", "gemm_xkv", "xattn_fwd", "gemm_xo"}
    phase_ms = {"fwd_ms": round(sum(v for k, v in step_ms.items() if k in fwd_names), 4),
                "bwd_ms": round(sum(v for k, v in step_ms.items() if k not in fwd_names and k != "adafactor"), 4),
                "adafactor_ms": round(step_ms.get("adafactor", 0.0), 4)}
    # HBM-bound steps: algorithmic bytes per step (2-byte activations; Adafactor: read G, read W, write W
    # in float32 plus the refreshed bf16 copy)
    Tn, dn_ = cfg.tokens, cfg.d_model
    n_params = sum(int(v.numel()) for v in w.values())
    if model_opt is not None:  # the whole model's tensors; unfactored ones also read and write their full second moment
        n_params = sum(int(t["param"].numel()) * (1.0 if t["factored"] else 22.0 / 14.0) for t in model_opt)
    # launches of each norm kernel per step
    n_norm = 2 * sc.n_layers + 1 if sc is not None else (3 if decoder else 2)
    if ec is not None:
        n_norm = 0  # encoder and decoder norms differ in size: no per-step byte count
    hbm_bytes = {"rmsnorm_fwd": n_norm * (2.0 * Tn * dn_ * 2 + 4.0 * Tn), "rmsnorm_bwd": n_norm * (4.0 * Tn * dn_ * 2),
                 "adafactor": 14.0 * n_params}
    if ec is not None:
        hbm_bytes = {"xent_rows": 2.0 * Tn * ec.vocab * 2, "adafactor": 14.0 * n_params}
    if sc is not None:
        # the loss reads every logit once and writes its gradient over it; the lookup copies T rows, its
        # gradient reads T rows and adds them into float32 rows (read + write)
        hbm_bytes.update({"xent_rows": 2.0 * Tn * sc.vocab * 2, "embed_fwd": 2.0 * Tn * dn_ * 2,
                          "embed_bwd": Tn * dn_ * (2.0 + 8.0)})

    # ---- what this machine sustains with nothing in the way (context for the fractions below)
    sink = torch.zeros(256, dtype=torch.float32, device=dev)
    machine = {}
    for label, rnd in (("mfma_loop_const_operands_tflops", False), ("mfma_loop_random_operands_tflops", True)):
        P.t5_mfma_peak_probe(1024, 2000, rnd, sink)
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        fl = P.t5_mfma_peak_probe(1024, 4000, rnd, sink)
        e1.record(); torch.cuda.synchronize()
        machine[label] = round(fl / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    src = torch.empty(1 << 29, dtype=torch.uint8, device=dev).zero_()
    dst = torch.empty_like(src)
    dst.copy_(src); torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record(); torch.cuda.synchronize()
    machine["copy_read_plus_write_gbs"] = round(5 * 2.0 * (1 << 29) / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    del src, dst
    mfma_steps = {k: v for k, v in per_kernel.items() if k in flops}
    dom = max(mfma_steps, key=lambda k: mfma_steps[k]["avg_ms"] * mfma_steps[k]["launches_per_step"])
    dom_tflops = flops[dom] / (per_kernel[dom]["avg_ms"] * 1e-3) / 1e12
    # HBM bytes per launch of that kernel come from committed rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE,
    # scaled by the same counters on a plain copy); bench.py cannot collect counters itself.
    traffic = None
    traffic_detail = None
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as fh:
            traffic_detail = json.load(fh).get(cfg.name, {}).get(dom)
        if traffic_detail is not None:
            traffic = int(traffic_detail["read_bytes"]) + int(traffic_detail["write_bytes"])
    except (OSError, ValueError, KeyError, TypeError):
        traffic = None
    roofline = {"bound": "mfma", "kernel": dom, "achieved": round(dom_tflops, 2), "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(dom_tflops / PEAK_BF16_TFLOPS, 4), "traffic": traffic,
                "traffic_unit": "HBM bytes per launch (read + write)", "traffic_detail": traffic_detail,
                "avg_ms": round(per_kernel[dom]["avg_ms"], 4), "flop_per_launch": flops[dom]}
    roofline["frac_of_measured_mfma_loop"] = round(dom_tflops / machine["mfma_loop_random_operands_tflops"], 4)
    for k, v in per_kernel.items():
        if k in flops and v["avg_ms"] > 0:
            v["tflops"] = round(flops[k] / (v["avg_ms"] * 1e-3) / 1e12, 1)
            v["bound"] = "mfma"
            v["frac"] = round(v["tflops"] / PEAK_BF16_TFLOPS, 4)
        elif k in hbm_bytes and step_ms[k] > 0:
            v["gbs"] = round(hbm_bytes[k] / (step_ms[k] * 1e-3) / 1e9, 1)
            v["bound"] = "hbm"
            v["frac"] = round(v["gbs"] / PEAK_HBM_GBS, 4)
        v["avg_ms"] = round(v["avg_ms"], 4)

    out = {
        "metric": "T5 block fwd+bwd tokens/s and TFLOP/s (bf16) + % MFMA peak, 1 MI355X",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "launch": ("hip graph replay" if args.graph else "eager") + (", weight gradients on a second stream" if args.overlap else ""),
        "config": {"workload": args.workload, "batch": cfg.batch, "seq_len": cfg.seq, "d_model": cfg.d_model,
                   "n_heads": cfg.n_heads, "d_kv": cfg.d_kv, "d_ff": cfg.d_ff, "causal": cfg.causal,
                   "enc_seq_len": cfg.enc_seq, "dropout_rate": cfg.dropout_rate, "deterministic": bool(cfg.deterministic), "attn_scale": cfg.attn_scale,
                   "adafactor": cfg.adafactor, "passes": "fwd+bwd" + ("+adafactor" if cfg.adafactor or (args.optimizer and (sc is not None or ec is not None)) else ""),
                   **({"n_layers": sc.n_layers, "vocab": sc.vocab, "tied_logits": sc.tied_logits, "remat": sc.remat,
                       "z_loss": sc.z_loss} if sc is not None else {}),
                   **({"n_enc_layers": ec.n_enc_layers, "n_dec_layers": ec.n_dec_layers, "vocab": ec.vocab,
                       "enc_seq_len": ec.enc_block.seq, "tokens_counted": "encoder + decoder positions",
                       "tied_logits": ec.tied_logits, "remat": ec.remat, "z_loss": ec.z_loss} if ec is not None else {})},
        "model_tflops": round(model_tflops, 2), "frac_of_mfma_peak": round(model_tflops / PEAK_BF16_TFLOPS, 4),
        "roofline": roofline, **phase_ms, "machine": machine, "per_kernel": per_kernel,
    }
    if not args.no_cpu_baseline:
        sb = args.cpu_sample_batch
        if sb <= 0:
            # float64 numpy sustains roughly 270 GFLOP/s on the box's 16 host cores (measured: c5_xl at batch 6 takes 8.3 s); aim near 15 s
            per_seq = total_model_flops / cfg.batch
            sb = int(max(1, min(cfg.batch, 15.0 * 270e9 / per_seq)))
        out["cpu_baseline"] = (cpu_baseline_stack(sc, sb) if sc is not None else
                               cpu_baseline_encdec(ec, sb) if ec is not None else cpu_baseline(cfg, sb))
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
