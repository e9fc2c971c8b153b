"""The FLOP counts behind the reported TFLOP/s, pinned three ways (CPU only).

1. The closed form of synth_inputs.BlockConfig.model_flops against the matrix products the oracle really
   performs: the oracle runs on an ndarray subclass that counts 2*M*N*K of every matmul it executes.
2. The closed form against the per-token formula written out here (projections 8 d I, attention 4 S I, gated MLP
   6 d F; backward twice the forward) at the named shapes.
3. bench.py's per-step table sums to the same total, so that per-kernel rates and the whole-step rate use one
   accounting.
"""
import dataclasses

import numpy as np
import pytest

import bench
import synth_inputs as SI
from oracle import t5_oracle as O


class Counting(np.ndarray):
    """ndarray whose matmuls are counted (2 * rows * cols * contraction per product, batched)."""
    flops = 0.0

    def __array_ufunc__(self, ufunc, method, *inputs, out=None, **kw):
        raw = [np.asarray(a).view(np.ndarray) if isinstance(a, np.ndarray) else a for a in inputs]
        if out is not None:
            kw["out"] = tuple(np.asarray(o).view(np.ndarray) for o in out)
        res = getattr(ufunc, method)(*raw, **kw)
        if ufunc is np.matmul and method == "__call__":
            a, b = raw[0], raw[1]
            r = np.asarray(res)
            Counting.flops += 2.0 * r.size * a.shape[-1]
        if isinstance(res, tuple):
            return tuple(np.asarray(x).view(Counting) if isinstance(x, np.ndarray) else x for x in res)
        return np.asarray(res).view(Counting) if isinstance(res, np.ndarray) else res


def _counted(cfg):
    w = {k: np.asarray(v, dtype=np.float64).view(Counting) for k, v in SI.make_weights(cfg).items()}
    x, dy = SI.make_activations(cfg)
    x, dy = np.asarray(x, dtype=np.float64).view(Counting), np.asarray(dy, dtype=np.float64).view(Counting)
    Counting.flops = 0.0
    y, saved = O.block_fwd(cfg, x, w)
    fwd = Counting.flops
    O.block_bwd(cfg, dy, w, saved)
    return fwd, Counting.flops - fwd


@pytest.mark.parametrize("causal", [False, True])
def test_closed_form_matches_the_products_the_oracle_performs(causal):
    cfg = dataclasses.replace(SI.CONFIGS["c1_tiny_f32"], batch=3, seq=40, causal=causal)
    fwd, bwd = _counted(cfg)
    # the oracle forms the full score matrix, masked or not: compare with the full count
    per_tok = cfg.fwd_flops_per_token(causal_half=False)
    assert fwd == pytest.approx(per_tok * cfg.tokens, rel=1e-12)
    assert bwd == pytest.approx(2.0 * per_tok * cfg.tokens, rel=1e-12)
    assert cfg.model_flops(causal_half=False) == pytest.approx(fwd + bwd, rel=1e-12)
    if causal:  # the causal count drops half of the two attention products and nothing else
        full, half = cfg.model_flops(causal_half=False), cfg.model_flops(causal_half=True)
        assert full - half == pytest.approx(3.0 * 2.0 * cfg.seq * cfg.inner * cfg.tokens, rel=1e-12)


def test_decoder_layer_closed_form_matches_the_oracle():
    cfg = dataclasses.replace(SI.CONFIGS["c1_tiny_f32"], batch=2, seq=24, causal=True, enc_seq=56)
    w = {k: np.asarray(v, dtype=np.float64).view(Counting) for k, v in SI.make_weights(cfg).items()}
    x, dy = SI.make_activations(cfg)
    enc = SI.make_encoder_output(cfg)
    as_c = lambda a: np.asarray(a, dtype=np.float64).view(Counting)
    Counting.flops = 0.0
    y, saved = O.decoder_block_fwd(cfg, as_c(x), as_c(enc), w)
    fwd = Counting.flops
    O.decoder_block_bwd(cfg, as_c(dy), w, saved)
    bwd = Counting.flops - fwd
    per_tok = cfg.fwd_flops_per_token(causal_half=False)
    assert fwd == pytest.approx(per_tok * cfg.tokens, rel=1e-12)
    assert bwd == pytest.approx(2.0 * per_tok * cfg.tokens, rel=1e-12)


@pytest.mark.parametrize("name, expect", [("c2_small", 5.41e11), ("c3_base", 3.09e12), ("c4_gpt_causal", 1.031e13),
                                          ("c5_xl", 1.031e13)])
def test_named_shapes(name, expect):
    c = SI.CONFIGS[name]
    d, I, S, F, T = c.d_model, c.n_heads * c.d_kv, c.seq, c.d_ff, c.batch * c.seq
    attn = 4 * S * I // (2 if c.causal else 1)
    by_hand = 3 * T * (8 * d * I + attn + 6 * d * F)
    assert c.model_flops() == by_hand
    assert by_hand == pytest.approx(expect, rel=2e-3)


@pytest.mark.parametrize("name", ["c2_small", "c3_base", "c4_gpt_causal", "c5_xl", "c6_dec_base", "c7_xl_tp8_share"])
def test_per_step_table_sums_to_the_model_count(name):
    c = SI.CONFIGS[name]
    assert sum(bench.gemm_step_flops(c).values()) == pytest.approx(c.model_flops(), rel=1e-12)
