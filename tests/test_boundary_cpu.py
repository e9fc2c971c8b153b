"""Host-only checks of the C ABI: the library loads, exports every function the header declares,
and rejects bad arguments before touching the GPU (so these run on a machine without one)."""
import ctypes as C
import os
import re

import pytest

import synth_inputs as SI
import paper_2203_17189_amd as P
from paper_2203_17189_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    src = open(os.path.join(ROOT, "include", "t5mi.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"\b([a-z0-9_]+)\s*\([^;{}]*\)\s*;", src)
    return sorted(set(names))


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert {"t5_relpos_bucket", "t5_block_fwd", "t5_block_bwd", "adafactor_step"} <= set(names)
    lib = P.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    assert P.t5_status_string(0) == "ok"
    assert "workspace" in P.t5_status_string(4)


def test_size_queries():
    for cfg in SI.CONFIGS.values():
        assert P.t5_block_stash_bytes(cfg) > 0 and P.t5_block_workspace_bytes(cfg) > 0
    bad = SI.CONFIGS["c1_tiny_f32"].with_batch(0)
    assert P.t5_block_stash_bytes(bad) == 0 and P.t5_block_workspace_bytes(bad) == 0
    assert P.adafactor_workspace_bytes(0, 5, True) == 0
    assert P.adafactor_workspace_bytes(64, 64, True) > 0


def test_relpos_validation():
    lib = P.lib()
    one = C.c_int32(0)
    p = C.cast(C.pointer(one), C.c_void_p)   # never dereferenced: every case fails validation first
    assert lib.t5_relpos_bucket(p, p, -1, 1, 32, 128, None) == 2
    assert lib.t5_relpos_bucket(p, p, 1, 1, 31, 128, None) == 2      # odd buckets, bidirectional
    assert lib.t5_relpos_bucket(p, p, 1, 1, 32, 8, None) == 2        # max_distance inside exact range
    assert lib.t5_relpos_bucket(p, p, 1, 0, 1, 128, None) == 2
    assert lib.t5_relpos_bucket(p, p, 1, 0, 512, 100000, None) == 3  # too many logarithmic buckets
    assert lib.t5_relpos_bucket(None, p, 1, 1, 32, 128, None) == 1
    assert lib.t5_relpos_bucket(None, None, 0, 1, 32, 128, None) == 0  # empty input is a no-op


def test_block_validation():
    lib = P.lib()
    cfg = B._cfg_struct(SI.CONFIGS["c1_tiny_f32"])
    dummy = C.c_void_p(4096)                  # non-null placeholder; validation fails before any use
    w = B._Weights(*([4096] * 10))
    g = B._Grads(*([4096] * 10))
    assert lib.t5_block_fwd(None, dummy, C.byref(w), dummy, dummy, dummy, 1 << 30, None) == 1
    assert lib.t5_block_fwd(C.byref(cfg), None, C.byref(w), dummy, dummy, dummy, 1 << 30, None) == 1
    w_missing = B._Weights(*([4096] * 9 + [None]))
    assert lib.t5_block_fwd(C.byref(cfg), dummy, C.byref(w_missing), dummy, dummy, dummy, 1 << 30, None) == 1
    assert lib.t5_block_fwd(C.byref(cfg), dummy, C.byref(w), dummy, dummy, dummy, 16, None) == 4
    assert lib.t5_block_bwd(C.byref(cfg), dummy, dummy, C.byref(w), dummy, dummy, C.byref(g), 0, dummy, 16,
                            None) == 4
    g_missing = B._Grads(*([None] + [4096] * 9))
    assert lib.t5_block_bwd(C.byref(cfg), dummy, dummy, C.byref(w), dummy, dummy, C.byref(g_missing), 0,
                            dummy, 1 << 30, None) == 1
    bad = B._cfg_struct(SI.CONFIGS["c1_tiny_f32"])
    bad.d_kv = 0
    assert lib.t5_block_fwd(C.byref(bad), dummy, C.byref(w), dummy, dummy, dummy, 1 << 30, None) == 2
    bad = B._cfg_struct(SI.CONFIGS["c1_tiny_f32"])
    bad.dtype = 7
    assert lib.t5_block_fwd(C.byref(bad), dummy, C.byref(w), dummy, dummy, dummy, 1 << 30, None) == 3
    bad = B._cfg_struct(SI.CONFIGS["c1_tiny_f32"])
    bad.num_buckets = 33
    assert lib.t5_block_fwd(C.byref(bad), dummy, C.byref(w), dummy, dummy, dummy, 1 << 30, None) == 2


def test_decoder_block_validation():
    lib = P.lib()
    cfg = B._cfg_struct(SI.CONFIGS["c1_tiny_f32"])
    dummy = C.c_void_p(4096)
    w = B._Weights(*([4096] * 10))
    g = B._Grads(*([4096] * 10))
    xw = B._CrossWeights(*([4096] * 5))
    xg = B._CrossGrads(*([4096] * 5))
    dec = SI.CONFIGS["c6_dec_base"]
    assert P.t5_decoder_block_stash_bytes(dec) > P.t5_block_stash_bytes(dec)
    assert P.t5_decoder_block_workspace_bytes(dec) > P.t5_block_workspace_bytes(dec)
    assert lib.t5_decoder_block_stash_bytes(C.byref(cfg), 0) == 0
    assert lib.t5_decoder_block_workspace_bytes(C.byref(cfg), -3) == 0
    fwd = lambda c, es, x, enc, ww, xx, nbytes: lib.t5_decoder_block_fwd(c, es, x, enc, ww, xx, dummy, dummy, dummy,
                                                                      nbytes, None)
    big = 1 << 30
    assert fwd(None, 8, dummy, dummy, C.byref(w), C.byref(xw), big) == 1
    assert fwd(C.byref(cfg), 0, dummy, dummy, C.byref(w), C.byref(xw), big) == 2
    assert fwd(C.byref(cfg), 8, dummy, None, C.byref(w), C.byref(xw), big) == 1
    assert fwd(C.byref(cfg), 8, dummy, dummy, C.byref(w), None, big) == 1
    assert fwd(C.byref(cfg), 8, dummy, dummy, C.byref(w), C.byref(B._CrossWeights(*([4096] * 4 + [None]))), big) == 1
    assert fwd(C.byref(cfg), 8, dummy, dummy, C.byref(w), C.byref(xw), 16) == 4
    bwd = lambda es, denc, gg, xgg, nbytes: lib.t5_decoder_block_bwd(C.byref(cfg), es, dummy, dummy, dummy, C.byref(w),
                                                                     C.byref(xw), dummy, dummy, denc, gg, xgg, 0,
                                                                     dummy, nbytes, None)
    assert bwd(8, dummy, C.byref(g), C.byref(xg), 16) == 4
    assert bwd(8, None, C.byref(g), C.byref(xg), big) == 1
    assert bwd(8, dummy, C.byref(g), None, big) == 1
    assert bwd(8, dummy, C.byref(g), C.byref(B._CrossGrads(*([None] + [4096] * 4))), big) == 1
    assert bwd(0, dummy, C.byref(g), C.byref(xg), big) == 2


def test_stack_validation():
    lib = P.lib()
    sc = SI.STACK_CONFIGS["s1_lm_base"]
    assert P.t5_stack_workspace_bytes(sc) > sc.n_layers * P.t5_block_stash_bytes(sc.block)
    from dataclasses import replace
    assert P.t5_stack_workspace_bytes(replace(sc, remat=True)) < P.t5_stack_workspace_bytes(sc) // 2
    assert P.t5_stack_workspace_bytes(replace(sc, n_layers=0)) == 0
    assert P.t5_stack_workspace_bytes(replace(sc, vocab=1)) == 0
    cs = B._stack_cfg_struct(replace(sc, n_layers=2))
    dummy = C.c_void_p(4096)
    lw = (B._Weights * 2)(B._Weights(*([4096] * 10)), B._Weights(*([4096] * 9 + [None])))
    ok_lw = (B._Weights * 2)(B._Weights(*([4096] * 10)), B._Weights(*([4096] * 10)))
    mk = lambda layers, emb=4096, out=4096: B._StackWeights(emb, 4096, layers, 4096, out)
    call = lambda c, tok, wts, loss, grads, nbytes: lib.t5_stack_loss_and_grad(c, tok, dummy, wts, loss, grads, 0,
                                                                               dummy, nbytes, None)
    big = 1 << 40
    assert call(None, dummy, C.byref(mk(ok_lw)), dummy, None, big) == 1
    assert call(C.byref(cs), None, C.byref(mk(ok_lw)), dummy, None, big) == 1
    assert call(C.byref(cs), dummy, C.byref(mk(ok_lw)), None, None, big) == 1
    assert call(C.byref(cs), dummy, C.byref(mk(lw)), dummy, None, big) == 1              # a layer lacks wo_ff
    assert call(C.byref(cs), dummy, C.byref(mk(ok_lw, out=None)), dummy, None, big) == 1  # untied needs logits_w
    assert call(C.byref(cs), dummy, C.byref(mk(ok_lw)), dummy, None, 1024) == 4
    lg = (B._Grads * 2)(B._Grads(*([4096] * 10)), B._Grads(*([4096] * 10)))
    bad_g = B._StackGrads(None, 4096, lg, 4096, 4096)
    assert call(C.byref(cs), dummy, C.byref(mk(ok_lw)), dummy, C.byref(bad_g), big) == 1
    neg = B._stack_cfg_struct(replace(sc, z_loss=-1.0))
    assert call(C.byref(neg), dummy, C.byref(mk(ok_lw)), dummy, None, big) == 2
    tied = B._stack_cfg_struct(replace(sc, n_layers=2, tied_logits=True))
    assert call(C.byref(tied), dummy, C.byref(mk(ok_lw, out=None)), dummy, None, 1024) == 4   # tied: logits_w not needed


def test_encdec_validation():
    lib = P.lib()
    from dataclasses import replace
    ec = SI.ENCDEC_CONFIGS["e1_t5_base"]
    assert P.t5_encdec_workspace_bytes(ec) > 0
    assert P.t5_encdec_workspace_bytes(replace(ec, remat=True)) < P.t5_encdec_workspace_bytes(ec)
    assert P.t5_encdec_workspace_bytes(replace(ec, enc_block=replace(ec.enc_block, causal=True))) == 0
    assert P.t5_encdec_workspace_bytes(replace(ec, dec_block=replace(ec.dec_block, causal=False))) == 0
    assert P.t5_encdec_workspace_bytes(replace(ec, enc_block=replace(ec.enc_block, d_model=512))) == 0
    assert P.t5_encdec_workspace_bytes(replace(ec, n_dec_layers=0)) == 0
    small = replace(ec, n_enc_layers=1, n_dec_layers=1)
    cs = B._encdec_cfg_struct(small)
    dummy = C.c_void_p(4096)
    lw = (B._Weights * 1)(B._Weights(*([4096] * 10)))
    xw = (B._CrossWeights * 1)(B._CrossWeights(*([4096] * 5)))
    wts = B._EncDecWeights(4096, 4096, lw, 4096, 4096, lw, xw, 4096, 4096)
    call = lambda w_, nbytes: lib.t5_encdec_loss_and_grad(C.byref(cs), dummy, dummy, dummy, w_, dummy, None, 0, dummy,
                                                          nbytes, None)
    assert call(C.byref(wts), 1024) == 4
    no_cross = B._EncDecWeights(4096, 4096, lw, 4096, 4096, lw, None, 4096, 4096)
    assert call(C.byref(no_cross), 1 << 40) == 1
    bad_x = (B._CrossWeights * 1)(B._CrossWeights(*([4096] * 4 + [None])))
    assert call(C.byref(B._EncDecWeights(4096, 4096, lw, 4096, 4096, lw, bad_x, 4096, 4096)), 1 << 40) == 1
    assert call(C.byref(B._EncDecWeights(4096, None, lw, 4096, 4096, lw, xw, 4096, 4096)), 1 << 40) == 1
    assert lib.t5_encdec_loss_and_grad(C.byref(cs), None, dummy, dummy, C.byref(wts), dummy, None, 0, dummy, 1 << 40,
                                       None) == 1


def test_adafactor_validation():
    lib = P.lib()
    dummy = C.c_void_p(4096)
    ok = B._AfCfg(0.01, 0.8, 1e-30, 1e-3, 1.0, 1, 1)
    assert lib.adafactor_step(dummy, dummy, dummy, dummy, None, 8, 8, 1, None, None, dummy, 1 << 20, None) == 1
    assert lib.adafactor_step(dummy, dummy, dummy, dummy, None, 0, 8, 1, C.byref(ok), None, dummy, 1 << 20,
                              None) == 2
    step0 = B._AfCfg(0.01, 0.8, 1e-30, 1e-3, 1.0, 1, 0)
    assert lib.adafactor_step(dummy, dummy, dummy, dummy, None, 8, 8, 1, C.byref(step0), None, dummy, 1 << 20,
                              None) == 2
    assert lib.adafactor_step(dummy, dummy, None, dummy, None, 8, 8, 1, C.byref(ok), None, dummy, 1 << 20,
                              None) == 1
    assert lib.adafactor_step(dummy, dummy, None, None, None, 8, 8, 0, C.byref(ok), None, dummy, 1 << 20,
                              None) == 1
    assert lib.adafactor_step(dummy, dummy, dummy, dummy, None, 8, 8, 1, C.byref(ok), None, dummy, 8, None) == 4


def test_adafactor_variant_validation():
    lib = P.lib()
    dummy = C.c_void_p(4096)
    mom = B._AfCfg(0.01, 0.8, 1e-30, 1e-3, 1.0, 1, 1, 0.9, 0.0)
    assert lib.adafactor_step(dummy, dummy, dummy, dummy, None, 8, 8, 1, C.byref(mom), None, dummy, 1 << 20,
                              None) == 3      # the single-tensor call has no momentum buffer
    arr = (B._AfTensor * 1)()
    arr[0] = B._AfTensor(4096, 4096, 4096, 4096, None, 8, 8, 1, None, None)
    need = lib.adafactor_multi_workspace_bytes(arr, 1)
    assert lib.adafactor_step_multi(arr, 1, C.byref(mom), dummy, need, None) == 1     # beta1 > 0 without m
    for bad in (B._AfCfg(0.01, 0.8, 1e-30, 1e-3, 1.0, 1, 1, 1.0, 0.0), B._AfCfg(0.01, 0.8, 1e-30, 1e-3, 1.0, 1, 1, -0.1, 0.0),
                B._AfCfg(0.01, 0.8, 1e-30, 1e-3, 1.0, 1, 1, 0.0, -1.0)):
        assert lib.adafactor_step_multi(arr, 1, C.byref(bad), dummy, need, None) == 2
        assert lib.adafactor_step(dummy, dummy, dummy, dummy, None, 8, 8, 1, C.byref(bad), None, dummy, 1 << 20,
                                  None) == 2


def test_adafactor_multi_validation():
    lib = P.lib()
    ok = B._AfCfg(0.01, 0.8, 1e-30, 1e-3, 1.0, 1, 1)
    arr = (B._AfTensor * 2)()
    arr[0] = B._AfTensor(4096, 4096, 4096, 4096, None, 8, 8, 1, None)
    arr[1] = B._AfTensor(4096, 4096, None, None, 4096, 1, 16, 0, None)
    need = lib.adafactor_multi_workspace_bytes(arr, 2)
    assert need == lib.adafactor_workspace_bytes(8, 8, 1) + lib.adafactor_workspace_bytes(1, 16, 0)
    dummy = C.c_void_p(4096)
    assert lib.adafactor_step_multi(arr, 2, None, dummy, need, None) == 1
    assert lib.adafactor_step_multi(None, 2, C.byref(ok), dummy, need, None) == 1
    assert lib.adafactor_step_multi(arr, 0, C.byref(ok), dummy, need, None) == 2
    assert lib.adafactor_step_multi(arr, (1 << 16) + 1, C.byref(ok), dummy, need, None) == 3
    many = (B._AfTensor * 40)(*([arr[0]] * 40))         # groups of 16: the workspace is the largest group's
    assert lib.adafactor_multi_workspace_bytes(many, 40) == 16 * lib.adafactor_workspace_bytes(8, 8, 1)
    assert lib.adafactor_step_multi(arr, 2, C.byref(ok), dummy, need - 1, None) == 4
    assert lib.adafactor_step_multi(arr, 2, C.byref(ok), None, need, None) == 1
    bad = (B._AfTensor * 1)()
    bad[0] = B._AfTensor(4096, 4096, None, 4096, None, 8, 8, 1, None)   # factored without v_row
    assert lib.adafactor_step_multi(bad, 1, C.byref(ok), dummy, 1 << 20, None) == 1
    bad[0] = B._AfTensor(4096, 4096, 4096, 4096, None, 0, 8, 1, None)
    assert lib.adafactor_step_multi(bad, 1, C.byref(ok), dummy, 1 << 20, None) == 2
    assert lib.t5_mfma_peak_probe(0, 1, 0, dummy, None) == 2
    assert lib.t5_mfma_peak_probe(1, 1, 0, None, None) == 1


def test_gemm_validation():
    lib = P.lib()
    dummy = C.c_void_p(4096)
    assert lib.t5_gemm_bf16(dummy, dummy, dummy, 0, 64, 64, 64, 64, 64, 1, 1, None) == 2
    assert lib.t5_gemm_bf16(None, dummy, dummy, 64, 64, 64, 64, 64, 64, 1, 1, None) == 1
    assert lib.t5_gemm_bf16(dummy, dummy, dummy, 64, 64, 72, 72, 72, 64, 1, 1, None) == 3   # K % 64
    assert lib.t5_gemm_bf16(dummy, dummy, dummy, 64, 64, 64, 64, 64, 64, 1, 0, None) == 3   # mixed layouts


def test_dropout_validation():
    lib = P.lib()
    dummy = C.c_void_p(4096)
    w = B._Weights(*([4096] * 10))
    keep = lambda seed, site, rate, rows, cols, out: lib.t5_dropout_keep(C.c_uint64(seed), site, C.c_float(rate), rows,
                                                                         cols, out, None)
    assert keep(1, 1, 0.1, 0, 16, None) == 0            # nothing to write
    assert keep(1, 1, 0.1, 4, 4, None) == 1
    assert keep(1, 1, 1.0, 4, 4, dummy) == 2
    assert keep(1, 1, -0.5, 4, 4, dummy) == 2
    assert keep(1, 1, float("nan"), 4, 4, dummy) == 2
    assert keep(1, 1, 0.1, -1, 4, dummy) == 2
    for rate in (1.0, -0.25, float("nan")):
        bad = B._cfg_struct(SI.CONFIGS["c1_tiny_f32"])
        bad.dropout_rate = rate
        assert lib.t5_block_fwd(C.byref(bad), dummy, C.byref(w), dummy, dummy, dummy, 1 << 30, None) == 2
    # the backward of a block with dropout needs room for the masked gradient copy
    from dataclasses import replace
    c1 = SI.CONFIGS["c1_tiny_f32"]
    assert P.t5_block_workspace_bytes(replace(c1, dropout_rate=0.5)) >= P.t5_block_workspace_bytes(c1)
    assert P.t5_block_stash_bytes(replace(c1, dropout_rate=0.5)) == P.t5_block_stash_bytes(c1)   # no mask is stored
