"""GPU parity: HIP path (through the C ABI) against the float64 oracle, element by element, on
shapes the oracle finishes in seconds."""
from dataclasses import replace

import numpy as np
import pytest
import torch

import synth_inputs as SI
from oracle import t5_oracle as O
from parity_util import (TOL_F32, block_floors, check_bf16, is_relu, make_case, rel_err,
                         run_block_gpu, to_np)

pytestmark = pytest.mark.gpu


def _P():
    import paper_2203_17189_amd as P
    return P


# ------------------------------------------------------------------ relative-position buckets
@pytest.mark.parametrize("bidir", [True, False])
@pytest.mark.parametrize("nb,md", [(32, 128), (16, 64), (8, 20), (64, 1000), (128, 4096)])
def test_relpos_bucket_bit_exact(bidir, nb, md):
    rp = np.arange(-5000, 5001, dtype=np.int32)
    got = _P().t5_relpos_bucket(torch.from_numpy(rp).cuda(), bidir, nb, md).cpu().numpy()
    want = O.relpos_bucket(rp, bidir, nb, md)
    assert np.array_equal(got.astype(np.int64), want)


def test_relpos_bucket_empty_and_large():
    P = _P()
    out = P.t5_relpos_bucket(torch.empty(0, dtype=torch.int32, device="cuda"), True)
    assert out.numel() == 0
    rng = np.random.default_rng(1)
    rp = rng.integers(-3000, 3000, size=1 << 20).astype(np.int32)
    rp[:4] = [-(2 ** 31) + 1, 2 ** 31 - 1, 0, -1]
    got = P.t5_relpos_bucket(torch.from_numpy(rp).cuda(), False).cpu().numpy()
    uniq = {int(v): O.relpos_bucket_scalar(int(v), False) for v in np.unique(rp)}
    want = np.array([uniq[int(v)] for v in rp])
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ float32 block (tiny config)
C1 = SI.CONFIGS["c1_tiny_f32"]


@pytest.mark.parametrize("cfg", [C1, replace(C1, causal=True, index=20),
                                 replace(C1, name="ragged", index=21, batch=3, seq=37, d_model=72, n_heads=3,
                                         d_kv=20, d_ff=100, attn_scale=0.25),
                                 replace(C1, name="long_causal", index=22, batch=1, seq=300, causal=True),
                                 replace(C1, name="relu_ff", index=23, mlp="relu"),
                                 replace(C1, name="erf_gelu_ff", index=24, mlp="geglu_erf", causal=True),
                                 replace(C1, name="relu_ff_ragged", index=25, batch=3, seq=37, d_model=72, n_heads=3,
                                         d_kv=20, d_ff=100, attn_scale=0.25, mlp="relu")])
def test_block_f32(cfg):
    w, x, dy = make_case(cfg)
    y, saved = O.block_fwd(cfg, x, w)
    dx, g = O.block_bwd(cfg, dy, w, saved)
    gy, gdx, gg = run_block_gpu(cfg, w, x, dy)
    assert rel_err(gy, y)[0] <= TOL_F32[0], ("y", rel_err(gy, y))
    assert rel_err(gdx, dx)[0] <= TOL_F32[0], ("dx", rel_err(gdx, dx))
    for name in g:
        assert rel_err(gg[name], g[name])[0] <= TOL_F32[0], (name, rel_err(gg[name], g[name]))


def test_block_f32_accumulate_flag():
    P = _P()
    from parity_util import upload_case
    cfg = C1
    w, x, dy = make_case(cfg)
    dw, dx_in, ddy = upload_case(cfg, w, x, dy)
    y, stash = P.t5_block_fwd(cfg, dx_in, dw)
    _, g1 = P.t5_block_bwd(cfg, ddy, dx_in, dw, stash)
    g2 = {k: v.clone() for k, v in g1.items()}
    P.t5_block_bwd(cfg, ddy, dx_in, dw, stash, grads=g2, accumulate=True)
    torch.cuda.synchronize()
    for k in g1:
        np.testing.assert_allclose(to_np(g2[k]), 2 * to_np(g1[k]), rtol=1e-5, atol=1e-6)


# ------------------------------------------------------------------ Adafactor
@pytest.mark.parametrize("rows,cols,factored", [(64, 256, True), (70, 130, True), (513, 1027, True),
                                                (1, 64, False), (32, 4, False), (33, 7, False)])
def test_adafactor_three_steps(rows, cols, factored):
    P = _P()
    p, _ = SI.make_adafactor_case(rows, cols, seed=5)
    st = O.adafactor_zero_state(rows, cols, factored)
    dp = torch.from_numpy(p.astype(np.float32)).cuda()
    vr = torch.zeros(rows, device="cuda")
    vc = torch.zeros(cols, device="cuda")
    vf = torch.zeros(rows, cols, device="cuda")
    lp = torch.empty(rows, cols, dtype=torch.bfloat16, device="cuda")
    w = p
    for t in (1, 2, 3):
        _, g = SI.make_adafactor_case(rows, cols, seed=30 + t, grad_std=1e-2 * t)
        w, st = O.adafactor_step(w, g, st, step=t, lr=0.01, factored=factored)
        P.adafactor_step(dp, torch.from_numpy(g.astype(np.float32)).cuda(), step=t, lr=0.01, factored=factored,
                         v_row=vr, v_col=vc, v_full=vf, bf16_copy_out=lp)
        torch.cuda.synchronize()
        assert rel_err(to_np(dp), w)[0] <= 1e-5, (t, rel_err(to_np(dp), w))
        if factored:
            assert rel_err(to_np(vr), st["vr"])[0] <= 1e-5
            assert rel_err(to_np(vc), st["vc"])[0] <= 1e-5
        else:
            assert rel_err(to_np(vf), st["v"])[0] <= 1e-5
        assert torch.equal(lp, dp.to(torch.bfloat16))


@pytest.mark.parametrize("rows,cols,factored", [(513, 1027, True), (33, 7, False)])
def test_adafactor_resume_from_saved_state_is_bit_identical(rows, cols, factored):
    """Checkpoint / resume on the device path: steps 1..3 straight through against steps 1..2, the parameter and
    the second-moment state copied out to the host and into fresh device buffers (what a checkpoint restore
    does), then step 3: the update keeps no hidden state, so the results agree bit for bit."""
    P = _P()
    p, _ = SI.make_adafactor_case(rows, cols, seed=9)
    grads = [torch.from_numpy(SI.make_adafactor_case(rows, cols, seed=40 + t, grad_std=1e-2 * t)[1].astype(np.float32)).cuda()
             for t in (1, 2, 3)]

    def fresh(src=None):
        st = dict(param=torch.from_numpy(p.astype(np.float32)).cuda(), v_row=torch.zeros(rows, device="cuda"),
                  v_col=torch.zeros(cols, device="cuda"), v_full=torch.zeros(rows, cols, device="cuda"))
        if src is not None:
            st = {k: torch.from_numpy(v.cpu().numpy().copy()).cuda() for k, v in src.items()}   # through host memory
        return st

    def step(st, t):
        P.adafactor_step(st["param"], grads[t - 1], step=t, lr=0.01, factored=factored, v_row=st["v_row"],
                         v_col=st["v_col"], v_full=st["v_full"])

    straight = fresh()
    for t in (1, 2, 3):
        step(straight, t)
    first = fresh()
    for t in (1, 2):
        step(first, t)
    torch.cuda.synchronize()
    resumed = fresh(first)
    step(resumed, 3)
    torch.cuda.synchronize()
    for k in straight:
        assert torch.equal(straight[k], resumed[k]), k
    assert not torch.equal(first["param"], resumed["param"])


def test_adafactor_multi_matches_single_and_oracle():
    # one batched call over tensors of mixed shapes (vectorised and not, factored and not) gives, bit for
    # bit, what the per-tensor calls give, and both match the float64 oracle
    P = _P()
    shapes = [(64, 256, True), (70, 130, True), (513, 1027, True), (1, 64, False), (32, 4, False), (33, 7, False),
              (128, 384, True)]
    single, multi, ref = [], [], []
    for k, (rows, cols, fact) in enumerate(shapes):
        p, _ = SI.make_adafactor_case(rows, cols, seed=50 + k)
        for group in (single, multi):
            group.append(dict(param=torch.from_numpy(p.astype(np.float32)).cuda(), factored=fact,
                              v_row=torch.zeros(rows, device="cuda"), v_col=torch.zeros(cols, device="cuda"),
                              v_full=torch.zeros(rows, cols, device="cuda"),
                              bf16_copy_out=torch.empty(rows, cols, dtype=torch.bfloat16, device="cuda")))
        ref.append((p, O.adafactor_zero_state(rows, cols, fact)))
    for t in (1, 2, 3):
        gs = []
        for k, (rows, cols, fact) in enumerate(shapes):
            _, g = SI.make_adafactor_case(rows, cols, seed=300 + 10 * t + k, grad_std=1e-2 * t)
            gs.append(g)
            ref[k] = O.adafactor_step(ref[k][0], g, ref[k][1], step=t, lr=0.01, factored=fact)
        for k, d in enumerate(single):
            gd = torch.from_numpy(gs[k].astype(np.float32)).cuda()
            P.adafactor_step(d["param"], gd, step=t, lr=0.01, factored=d["factored"], v_row=d["v_row"],
                             v_col=d["v_col"], v_full=d["v_full"], bf16_copy_out=d["bf16_copy_out"])
        for k, d in enumerate(multi):
            d["grad"] = torch.from_numpy(gs[k].astype(np.float32)).cuda()
        P.adafactor_step_multi(multi, step=t, lr=0.01)
        torch.cuda.synchronize()
        for k, (a, b) in enumerate(zip(single, multi)):
            assert torch.equal(a["param"], b["param"]), (t, k)
            assert torch.equal(a["bf16_copy_out"], b["bf16_copy_out"]), (t, k)
            assert rel_err(to_np(b["param"]), ref[k][0])[0] <= 1e-5, (t, k)


def test_adafactor_multi_long_list():
    # 37 tensors in one call: three groups of up to 16, sharing the workspace; each equals the oracle
    P = _P()
    shapes = [(8 + 3 * k, 24 + 5 * (k % 7), k % 3 != 0) for k in range(37)]
    items, ref = [], []
    for k, (rows, cols, fact) in enumerate(shapes):
        p, g = SI.make_adafactor_case(rows, cols, seed=700 + k)
        items.append(dict(param=torch.from_numpy(p.astype(np.float32)).cuda(), grad=torch.from_numpy(g.astype(np.float32)).cuda(),
                          factored=fact, v_row=torch.zeros(rows, device="cuda"), v_col=torch.zeros(cols, device="cuda"),
                          v_full=torch.zeros(rows, cols, device="cuda")))
        ref.append(O.adafactor_step(p, g, O.adafactor_zero_state(rows, cols, fact), step=1, lr=0.01, factored=fact)[0])
    P.adafactor_step_multi(items, step=1, lr=0.01)
    torch.cuda.synchronize()
    for k, d in enumerate(items):
        assert rel_err(to_np(d["param"]), ref[k])[0] <= 1e-5, k


def test_adafactor_momentum_and_weight_decay():
    # momentum buffers and decoupled decay through the batched entry point, four steps, against the oracle;
    # weight decay alone also through the single-tensor entry point
    P = _P()
    shapes = [(64, 256, True), (70, 130, True), (1, 64, False), (33, 7, False)]
    beta1, wd, lr = 0.9, 0.05, 0.02
    dev, ref, single = [], [], []
    for k, (rows, cols, fact) in enumerate(shapes):
        p, _ = SI.make_adafactor_case(rows, cols, seed=80 + k)
        mk = lambda: dict(param=torch.from_numpy(p.astype(np.float32)).cuda(), factored=fact,
                          v_row=torch.zeros(rows, device="cuda"), v_col=torch.zeros(cols, device="cuda"),
                          v_full=torch.zeros(rows, cols, device="cuda"), m=torch.zeros(rows, cols, device="cuda"))
        dev.append(mk())
        single.append(mk())
        ref.append([(p, O.adafactor_zero_state(rows, cols, fact, momentum=True)),
                    (p, O.adafactor_zero_state(rows, cols, fact))])
    for t in (1, 2, 3, 4):
        for k, (rows, cols, fact) in enumerate(shapes):
            _, g = SI.make_adafactor_case(rows, cols, seed=800 + 10 * t + k, grad_std=1e-2 * t)
            ref[k][0] = O.adafactor_step(ref[k][0][0], g, ref[k][0][1], step=t, lr=lr, factored=fact, beta1=beta1,
                                         weight_decay=wd)
            ref[k][1] = O.adafactor_step(ref[k][1][0], g, ref[k][1][1], step=t, lr=lr, factored=fact, weight_decay=wd)
            dev[k]["grad"] = torch.from_numpy(g.astype(np.float32)).cuda()
            d = single[k]
            P.adafactor_step(d["param"], dev[k]["grad"], step=t, lr=lr, factored=fact, v_row=d["v_row"],
                             v_col=d["v_col"], v_full=d["v_full"], weight_decay=wd)
        P.adafactor_step_multi(dev, step=t, lr=lr, beta1=beta1, weight_decay=wd)
        torch.cuda.synchronize()
        for k in range(len(shapes)):
            assert rel_err(to_np(dev[k]["param"]), ref[k][0][0])[0] <= 1e-5, (t, k)
            assert rel_err(to_np(dev[k]["m"]), ref[k][0][1]["m"])[0] <= 1e-5, (t, k)
            assert rel_err(to_np(single[k]["param"]), ref[k][1][0])[0] <= 1e-5, (t, k)


# ------------------------------------------------------------------ bf16 block, small shapes
SMALL_BF16 = [
    SI.BlockConfig("bf16_enc", 30, batch=2, seq=128, d_model=128, n_heads=2, d_kv=64, d_ff=256,
                   attn_scale=64 ** -0.5),
    SI.BlockConfig("bf16_dec", 31, batch=2, seq=192, d_model=128, n_heads=2, d_kv=64, d_ff=256, causal=True,
                   attn_scale=64 ** -0.5),
    SI.BlockConfig("bf16_dec_mfma", 33, batch=2, seq=384, d_model=128, n_heads=2, d_kv=64, d_ff=256, causal=True,
                   attn_scale=64 ** -0.5),
    SI.BlockConfig("bf16_enc_dk128", 34, batch=1, seq=256, d_model=256, n_heads=2, d_kv=128, d_ff=320,
                   attn_scale=128 ** -0.5),
    SI.BlockConfig("bf16_dec_dk128", 35, batch=2, seq=256, d_model=128, n_heads=3, d_kv=128, d_ff=192, causal=True,
                   attn_scale=128 ** -0.5),
    SI.BlockConfig("bf16_enc_long", 36, batch=1, seq=1024, d_model=64, n_heads=1, d_kv=64, d_ff=64,
                   attn_scale=64 ** -0.5),
    SI.BlockConfig("bf16_ragged", 32, batch=1, seq=100, d_model=72, n_heads=3, d_kv=24, d_ff=136,
                   attn_scale=24 ** -0.5),
    # long rows: 32 query tiles and 64 key tiles per head, causal, 128 channels (the largest per-head problem of
    # the workloads is 2048 x 2048)
    SI.BlockConfig("bf16_dec_4096_dk128", 29, batch=1, seq=4096, d_model=128, n_heads=1, d_kv=128, d_ff=128, causal=True,
                   attn_scale=128 ** -0.5),
    # other bucket tables: the saturated bucket starts at a small offset (narrow per-diagonal window in
    # the dq kernel, most sub-tiles take the scalar path) or beyond the sequence (every sub-tile is
    # resolved per diagonal)
    SI.BlockConfig("bf16_enc_b8_d20", 37, batch=1, seq=512, d_model=128, n_heads=2, d_kv=64, d_ff=128,
                   num_buckets=8, max_distance=20, attn_scale=64 ** -0.5),
    SI.BlockConfig("bf16_dec_b8_d20", 38, batch=1, seq=384, d_model=128, n_heads=2, d_kv=64, d_ff=128, causal=True,
                   num_buckets=8, max_distance=20, attn_scale=64 ** -0.5),
    # feed-forward variants on the matrix-unit path: ungated ReLU (original T5) and gated exact GELU
    SI.BlockConfig("bf16_enc_relu", 26, batch=2, seq=256, d_model=128, n_heads=2, d_kv=64, d_ff=256,
                   attn_scale=64 ** -0.5, mlp="relu"),
    SI.BlockConfig("bf16_dec_erf", 27, batch=2, seq=128, d_model=128, n_heads=2, d_kv=64, d_ff=256, causal=True,
                   attn_scale=64 ** -0.5, mlp="geglu_erf"),
    SI.BlockConfig("bf16_relu_ragged", 28, batch=1, seq=100, d_model=72, n_heads=3, d_kv=24, d_ff=136,
                   attn_scale=24 ** -0.5, mlp="relu"),
    SI.BlockConfig("bf16_enc_b64_d1000", 39, batch=1, seq=384, d_model=128, n_heads=2, d_kv=64, d_ff=128,
                   num_buckets=64, max_distance=1000, attn_scale=64 ** -0.5),
    # sequence lengths that are not multiples of the attention tiles, on the matrix-unit attention kernels
    # (RAGGED_MFMA below asserts the path): T5's 114 decoder positions (shorter than one query tile), 200
    # (ragged 64-key and 128-query tiles), 1000 (eight tiles, the last one ragged), both directions and widths
    SI.BlockConfig("bf16_enc_s114", 20, batch=2, seq=114, d_model=128, n_heads=2, d_kv=64, d_ff=256,
                   attn_scale=64 ** -0.5),
    SI.BlockConfig("bf16_dec_s114", 21, batch=2, seq=114, d_model=128, n_heads=2, d_kv=64, d_ff=256, causal=True,
                   attn_scale=64 ** -0.5),
    SI.BlockConfig("bf16_enc_s200_dk128", 22, batch=1, seq=200, d_model=256, n_heads=2, d_kv=128, d_ff=320,
                   attn_scale=128 ** -0.5),
    SI.BlockConfig("bf16_dec_s200", 23, batch=2, seq=200, d_model=128, n_heads=3, d_kv=64, d_ff=256, causal=True,
                   attn_scale=64 ** -0.5),
    SI.BlockConfig("bf16_enc_s1000", 24, batch=1, seq=1000, d_model=64, n_heads=1, d_kv=64, d_ff=64,
                   attn_scale=64 ** -0.5),
    SI.BlockConfig("bf16_dec_s1000_dk128", 25, batch=1, seq=1000, d_model=128, n_heads=1, d_kv=128, d_ff=128, causal=True,
                   attn_scale=128 ** -0.5),
    SI.BlockConfig("bf16_enc_s33_b8_d20", 19, batch=2, seq=33, d_model=64, n_heads=1, d_kv=64, d_ff=64,
                   num_buckets=8, max_distance=20, attn_scale=64 ** -0.5),
    # the longest sequence the fused attention takes, less one: every tile count at its maximum, and a ragged tail
    # (the oracle and the floor model materialise 8191 x 8191 scores: about a minute on the host)
    SI.BlockConfig("bf16_dec_s8191", 18, batch=1, seq=8191, d_model=64, n_heads=1, d_kv=64, d_ff=64, causal=True,
                   dtype="bf16", attn_scale=64 ** -0.5),
]
RAGGED_MFMA = ("bf16_enc_s114", "bf16_dec_s114", "bf16_enc_s200_dk128", "bf16_dec_s200", "bf16_enc_s1000",
               "bf16_dec_s1000_dk128", "bf16_enc_s33_b8_d20", "bf16_dec_s8191")


def test_block_bf16_accumulate_flag():
    # weight gradients are cleared once per backward unless accumulate is set; with it, a second
    # backward adds its split-k partial sums on top of the first result
    P = _P()
    from parity_util import upload_case
    cfg = SMALL_BF16[2]
    w, x, dy = make_case(cfg)
    dw, dx_in, ddy = upload_case(cfg, w, x, dy)
    y, stash = P.t5_block_fwd(cfg, dx_in, dw)
    _, g1 = P.t5_block_bwd(cfg, ddy, dx_in, dw, stash)
    g2 = {k: v.clone() for k, v in g1.items()}
    P.t5_block_bwd(cfg, ddy, dx_in, dw, stash, grads=g2, accumulate=True)
    torch.cuda.synchronize()
    twice = {k: to_np(v).copy() for k, v in g2.items()}
    P.t5_block_bwd(cfg, ddy, dx_in, dw, stash, grads=g2)  # without the flag: overwrites
    torch.cuda.synchronize()
    for k in g1:
        a1 = to_np(g1[k])
        scale = np.abs(a1).max() + 1e-30
        assert np.abs(twice[k] - 2 * a1).max() <= 4e-5 * scale, ("accumulate", k)
        assert np.abs(to_np(g2[k]) - a1).max() <= 2e-5 * scale, ("overwrite", k)


@pytest.mark.parametrize("cfg", SMALL_BF16, ids=[c.name for c in SMALL_BF16])
def test_block_bf16_small(cfg):
    if cfg.name in RAGGED_MFMA:   # these must run the fused matrix-unit attention, forward and backward
        P = _P()
        assert P.t5_block_kernel_path(cfg) & (P.PATH_MFMA_ATTN_FWD | P.PATH_MFMA_ATTN_BWD) == \
            (P.PATH_MFMA_ATTN_FWD | P.PATH_MFMA_ATTN_BWD), P.t5_block_kernel_path(cfg)
    w, x, dy = make_case(cfg)
    y, saved = O.block_fwd(cfg, x, w)
    dx, g = O.block_bwd(cfg, dy, w, saved)
    gy, gdx, gg = run_block_gpu(cfg, w, x, dy)
    errs = {"y": rel_err(gy, y), "dx": rel_err(gdx, dx), **{k: rel_err(gg[k], g[k]) for k in g}}
    check_bf16(cfg.name, errs, block_floors(cfg, w, x, dy, (y, dx, g)), relu=is_relu(cfg))
