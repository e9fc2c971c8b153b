"""Seeded synthetic inputs for one T5.1.1-style Transformer block.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests/bench.  It holds shapes, seeds and random draws only: none of
the block's arithmetic lives here.

The paper (Sec. 4, "Example models") names the T5.1.1 and decoder-only
architectures but ships no dataset with the hot path, so every tensor is a
seeded Gaussian draw with the shapes of those models:
  activations x and upstream gradients dy ~ N(0, 1)
  projection weights ~ N(0, fan_in^-1/2)   (std, not variance)
  relative-position bias table ~ N(0, 0.1) (std)
  RMSNorm scales = 1
Draws are made in float64 on the host, then rounded once to the config's
storage dtype (round-to-nearest-even); those rounded values are what both the
oracle and the GPU consume, so input quantisation never enters a comparison.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np

BASE_SEED = 20220331
TENSOR_ORDER = ("x", "dy", "wq", "wk", "wv", "wo", "rel_table", "wi0", "wi1", "wo_ff",
                "ln1_scale", "ln2_scale",
                # decoder block (cross-attention over an encoder output); appended so that the
                # seeds of the tensors above never change
                "enc", "xq", "xk", "xv", "xo", "lnx_scale")


@dataclass(frozen=True)
class BlockConfig:
    name: str
    index: int            # position in the workload list; enters the seed
    batch: int
    seq: int
    d_model: int
    n_heads: int
    d_kv: int
    d_ff: int
    causal: bool = False
    dtype: str = "bf16"   # storage dtype of activations and weights: "f32" | "bf16"
    num_buckets: int = 32
    max_distance: int = 128
    rms_eps: float = 1e-6
    attn_scale: float = 1.0   # T5 convention: no 1/sqrt(d_kv) on the logits
    adafactor: bool = False
    enc_seq: int = 0          # > 0: decoder block, with a cross-attention sublayer over an encoder
                              # output of this length between self-attention and the MLP

    @property
    def inner(self) -> int:
        return self.n_heads * self.d_kv

    @property
    def tokens(self) -> int:
        return self.batch * self.seq

    def with_batch(self, batch: int) -> "BlockConfig":
        return replace(self, batch=batch)

    def fwd_flops_per_token(self, causal_half: bool = True) -> float:
        d, i, s, f = self.d_model, self.inner, self.seq, self.d_ff
        attn = 4.0 * s * i
        if self.causal and causal_half:
            attn *= 0.5
        cross = 0.0
        if self.enc_seq > 0:
            # per decoder token: q and o projections, scores and values over enc_seq keys; the k, v
            # projections of the enc_seq encoder tokens are spread over the seq decoder tokens
            cross = 4.0 * d * i + 4.0 * self.enc_seq * i + 4.0 * d * i * self.enc_seq / s
        return 8.0 * d * i + attn + cross + 6.0 * d * f

    def model_flops(self, causal_half: bool = True) -> float:
        """fwd+bwd model FLOPs (3x forward), whole batch."""
        return 3.0 * self.fwd_flops_per_token(causal_half) * self.tokens


CONFIGS = {
    "c1_tiny_f32": BlockConfig("c1_tiny_f32", 0, 2, 32, 64, 4, 16, 256, dtype="f32", adafactor=True),
    "c2_small": BlockConfig("c2_small", 1, 64, 512, 512, 6, 64, 1024),
    "c3_base": BlockConfig("c3_base", 2, 128, 512, 768, 12, 64, 2048, adafactor=True),
    "c4_gpt_causal": BlockConfig("c4_gpt_causal", 3, 16, 2048, 2048, 16, 128, 5120, causal=True),
    "c5_xl": BlockConfig("c5_xl", 4, 32, 1024, 2048, 32, 64, 5120, adafactor=True),
    # T5.1.1-Base decoder block: causal self-attention, cross-attention over 512 encoder positions, MLP
    "c6_dec_base": BlockConfig("c6_dec_base", 5, 128, 512, 768, 12, 64, 2048, causal=True, enc_seq=512),
}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float values to the nearest bf16 (ties to even); returns float32 holding bf16 values."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    bits = a32.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).reshape(a32.shape)


def bf16_bits(a32: np.ndarray) -> np.ndarray:
    """uint16 payload of float32 values that are already bf16-representable."""
    return (np.ascontiguousarray(a32, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def round_to_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_to_bf16(a).astype(np.float64)
    if dtype == "f32":
        return a.astype(np.float32).astype(np.float64)
    raise ValueError(dtype)


def _draw(cfg: BlockConfig, tensor: str, shape, std: float, seed_offset: int = 0) -> np.ndarray:
    seed = BASE_SEED + 1000 * cfg.index + TENSOR_ORDER.index(tensor) + 100000 * seed_offset
    g = np.random.default_rng(seed).standard_normal(shape) * std
    return round_to_dtype(g, cfg.dtype)


def make_weights(cfg: BlockConfig) -> dict:
    """Block weights as float64 arrays holding dtype-representable values."""
    d, i, f, h = cfg.d_model, cfg.inner, cfg.d_ff, cfg.n_heads
    w = {
        "ln1_scale": np.ones(d),
        "wq": _draw(cfg, "wq", (d, i), d ** -0.5),
        "wk": _draw(cfg, "wk", (d, i), d ** -0.5),
        "wv": _draw(cfg, "wv", (d, i), d ** -0.5),
        "wo": _draw(cfg, "wo", (i, d), i ** -0.5),
        "rel_table": _draw(cfg, "rel_table", (cfg.num_buckets, h), 0.1),
        "ln2_scale": np.ones(d),
        "wi0": _draw(cfg, "wi0", (d, f), d ** -0.5),
        "wi1": _draw(cfg, "wi1", (d, f), d ** -0.5),
        "wo_ff": _draw(cfg, "wo_ff", (f, d), f ** -0.5),
    }
    if cfg.enc_seq > 0:
        w.update({
            "lnx_scale": np.ones(d),
            "xq": _draw(cfg, "xq", (d, i), d ** -0.5),
            "xk": _draw(cfg, "xk", (d, i), d ** -0.5),
            "xv": _draw(cfg, "xv", (d, i), d ** -0.5),
            "xo": _draw(cfg, "xo", (i, d), i ** -0.5),
        })
    return w


def make_random_scales(cfg: BlockConfig, seed_offset: int = 7) -> dict:
    """Non-trivial RMSNorm scales (1 + 0.1 N(0,1)) for tests that must see the scale's gradient path."""
    out = {}
    for name in ("ln1_scale", "ln2_scale") + (("lnx_scale",) if cfg.enc_seq > 0 else ()):
        out[name] = round_to_dtype(1.0 + _draw(cfg, name, (cfg.d_model,), 0.1, seed_offset), cfg.dtype)
    return out


def make_activations(cfg: BlockConfig, seed_offset: int = 0) -> tuple:
    """(x, dy), each [batch, seq, d_model] float64 holding dtype-representable values."""
    shape = (cfg.batch, cfg.seq, cfg.d_model)
    return _draw(cfg, "x", shape, 1.0, seed_offset), _draw(cfg, "dy", shape, 1.0, seed_offset)


def make_encoder_output(cfg: BlockConfig, seed_offset: int = 0) -> np.ndarray:
    """Encoder output read by the decoder block's cross-attention: [batch, enc_seq, d_model] ~ N(0, 1)."""
    return _draw(cfg, "enc", (cfg.batch, cfg.enc_seq, cfg.d_model), 1.0, seed_offset)


def make_adafactor_case(rows: int, cols: int, seed: int, grad_std: float = 1e-2) -> tuple:
    """(param, grad) float64 arrays holding float32-representable values for a standalone optimizer test."""
    rng = np.random.default_rng(BASE_SEED + 7919 * seed + rows * 31 + cols)
    p = rng.standard_normal((rows, cols)) * (max(rows, 1) ** -0.5)
    g = rng.standard_normal((rows, cols)) * grad_std
    # column- and row-dependent gradient scale so the factored statistics are not flat
    g = g * (0.5 + rng.random((rows, 1))) * (0.5 + rng.random((1, cols)))
    return p.astype(np.float32).astype(np.float64), g.astype(np.float32).astype(np.float64)
