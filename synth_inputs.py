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
    mlp: str = "geglu_tanh"   # feed-forward: "geglu_tanh" (T5.1.1) | "geglu_erf" | "relu" (original T5, no gate)
    dropout_rate: float = 0.0 # > 0: training-time dropout at the four T5 sites of the block
    dropout_seed: int = 0     # 64-bit seed of the counter-based generator (a caller varies it per step and layer)
    deterministic: bool = False  # True: weight and bias-table gradients summed in a fixed order (bit-reproducible)
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
        return 8.0 * d * i + attn + cross + (4.0 if self.mlp == "relu" else 6.0) * d * f

    def model_flops(self, causal_half: bool = True) -> float:
        """fwd+bwd model FLOPs (3x forward), whole batch."""
        return 3.0 * self.fwd_flops_per_token(causal_half) * self.tokens


CONFIGS = {
    "c1_tiny_f32": BlockConfig("c1_tiny_f32", 0, 2, 32, 64, 4, 16, 256, dtype="f32", adafactor=True),
    "c2_small": BlockConfig("c2_small", 1, 64, 512, 512, 6, 64, 1024),
    "c3_base": BlockConfig("c3_base", 2, 128, 512, 768, 12, 64, 2048, adafactor=True),
    "c4_gpt_causal": BlockConfig("c4_gpt_causal", 3, 16, 2048, 2048, 16, 128, 5120, causal=True),
    "c5_xl": BlockConfig("c5_xl", 4, 32, 1024, 2048, 32, 64, 5120, adafactor=True),
    # One GPU's share of c5_xl under the paper's tensor model parallelism (Sec. 2.2) over 8 devices: heads
    # and feed-forward width split by 8 (4 heads, d_ff 640); the [T, d] outputs would be summed across devices
    "c7_xl_tp8_share": BlockConfig("c7_xl_tp8_share", 7, 32, 1024, 2048, 4, 64, 640),
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
    if cfg.mlp == "relu":
        del w["wi1"]
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


@dataclass(frozen=True)
class StackConfig:
    """A stack of n_layers identical blocks with token embedding, final norm, logits and loss
    (paper Sec. 4: the decoder-only model when block.causal, else an encoder-style stack)."""
    name: str
    block: BlockConfig
    n_layers: int
    vocab: int
    tied_logits: bool = False   # False: separate [d_model, vocab] output matrix (T5.1.1)
    z_loss: float = 1e-4
    remat: bool = False         # True: keep layer inputs only, recompute each layer in the backward

    def with_batch(self, batch: int) -> "StackConfig":
        return replace(self, block=self.block.with_batch(batch))

    def model_flops(self) -> float:
        """fwd+bwd model FLOPs of one step (3x forward; the recompute of remat is not counted)."""
        b = self.block
        return 3.0 * b.tokens * (self.n_layers * b.fwd_flops_per_token() + 2.0 * b.d_model * self.vocab)


STACK_CONFIGS = {
    # T5.1.1-Base widths as a 12-layer decoder-only language model over the 32128-entry T5 vocabulary
    "s1_lm_base": StackConfig("s1_lm_base", BlockConfig("s1_lm_base", 6, 32, 512, 768, 12, 64, 2048, causal=True),
                              n_layers=12, vocab=32128),
}


def make_stack_weights(sc: StackConfig) -> dict:
    """{"embedding", "rel_table" (shared by all layers), "final_scale", "logits_w" (absent when tied),
    "layers": [block weight dicts without rel_table]}; float64 holding dtype-representable values."""
    b = sc.block
    rng_seed = BASE_SEED + 1000 * b.index + 500
    emb = np.random.default_rng(rng_seed).standard_normal((sc.vocab, b.d_model))
    w = {"embedding": round_to_dtype(emb, b.dtype), "final_scale": np.ones(b.d_model), "layers": []}
    for l in range(sc.n_layers):
        lw = make_weights(replace(b, index=b.index + 37 * (l + 1), enc_seq=0))
        table = lw.pop("rel_table")
        if l == 0:
            w["rel_table"] = table
        w["layers"].append(lw)
    if not sc.tied_logits:
        out = np.random.default_rng(rng_seed + 1).standard_normal((b.d_model, sc.vocab)) * b.d_model ** -0.5
        w["logits_w"] = round_to_dtype(out, b.dtype)
    return w


def make_stack_random_scales(sc: StackConfig, w: dict) -> None:
    """In place: non-trivial RMSNorm scales for every layer and the final norm."""
    b = sc.block
    for l, lw in enumerate(w["layers"]):
        lw.update(make_random_scales(replace(b, index=b.index + 37 * (l + 1), enc_seq=0)))
    g = np.random.default_rng(BASE_SEED + 1000 * b.index + 502).standard_normal(b.d_model)
    w["final_scale"] = round_to_dtype(1.0 + 0.1 * g, b.dtype)


def make_tokens(sc: StackConfig, seed_offset: int = 0, ignore_fraction: float = 0.1) -> tuple:
    """(tokens, targets) int32 [batch, seq].  Token ids follow a Zipf-like law over the vocabulary
    (probability ~ 1 / (rank + 10)), as natural-language token streams do; targets are the next
    token of the same stream, and a fraction of them is -1 (padding positions that carry no loss)."""
    b = sc.block
    rng = np.random.default_rng(BASE_SEED + 1000 * b.index + 503 + 100000 * seed_offset)
    p = 1.0 / (np.arange(sc.vocab) + 10.0)
    p /= p.sum()
    perm = rng.permutation(sc.vocab)                      # rank -> token id
    stream = perm[rng.choice(sc.vocab, size=(b.batch, b.seq + 1), p=p)]
    tokens = stream[:, :-1].astype(np.int32)
    targets = stream[:, 1:].astype(np.int32)
    if ignore_fraction > 0:
        targets = np.where(rng.random(targets.shape) < ignore_fraction, -1, targets).astype(np.int32)
    return tokens, targets


@dataclass(frozen=True)
class EncDecConfig:
    """Encoder-decoder model (paper Sec. 4, T5.1.1): a bidirectional encoder stack and a causal decoder
    stack whose layers cross-attend to the encoder output; one token embedding for both."""
    name: str
    enc_block: BlockConfig     # causal False; seq = encoder length
    dec_block: BlockConfig     # causal True; seq = decoder length; enc_seq = encoder length
    n_enc_layers: int
    n_dec_layers: int
    vocab: int
    tied_logits: bool = False
    z_loss: float = 1e-4
    remat: bool = False

    def with_batch(self, batch: int) -> "EncDecConfig":
        return replace(self, enc_block=self.enc_block.with_batch(batch), dec_block=self.dec_block.with_batch(batch))

    def model_flops(self) -> float:
        e, d = self.enc_block, self.dec_block
        return 3.0 * (e.tokens * self.n_enc_layers * e.fwd_flops_per_token()
                      + d.tokens * (self.n_dec_layers * d.fwd_flops_per_token() + 2.0 * d.d_model * self.vocab))


def _encdec(name, index, batch, enc_seq, dec_seq, d, h, dk, f, le, ld, vocab, **kw):
    blk = dict(kw.pop("block", {}))
    e = BlockConfig(name + "_enc", index, batch, enc_seq, d, h, dk, f, causal=False, **blk)
    dcd = BlockConfig(name + "_dec", index + 1, batch, dec_seq, d, h, dk, f, causal=True, enc_seq=enc_seq, **blk)
    return EncDecConfig(name, e, dcd, le, ld, vocab, **kw)


ENCDEC_CONFIGS = {
    # T5.1.1-Base: 12 + 12 layers, 512 encoder positions, 114 decoder positions in pre-training
    "e1_t5_base": _encdec("e1_t5_base", 8, 32, 512, 114, 768, 12, 64, 2048, 12, 12, 32128),
}


def make_encdec_weights(ec: EncDecConfig) -> dict:
    e, d = ec.enc_block, ec.dec_block
    enc = make_stack_weights(StackConfig("enc", e, ec.n_enc_layers, ec.vocab, tied_logits=True))
    w = {"embedding": enc["embedding"], "enc_rel_table": enc["rel_table"], "enc_layers": enc["layers"],
         "enc_final_scale": np.ones(e.d_model), "dec_final_scale": np.ones(d.d_model), "dec_layers": []}
    for l in range(ec.n_dec_layers):
        lw = make_weights(replace(d, index=d.index + 37 * (l + 1)))
        table = lw.pop("rel_table")
        if l == 0:
            w["dec_rel_table"] = table
        w["dec_layers"].append(lw)
    if not ec.tied_logits:
        out = np.random.default_rng(BASE_SEED + 1000 * d.index + 501).standard_normal((d.d_model, ec.vocab))
        w["logits_w"] = round_to_dtype(out * d.d_model ** -0.5, d.dtype)
    return w


def make_encdec_random_scales(ec: EncDecConfig, w: dict) -> None:
    """In place: non-trivial RMSNorm scales everywhere."""
    e, d = ec.enc_block, ec.dec_block
    for l, lw in enumerate(w["enc_layers"]):
        lw.update(make_random_scales(replace(e, index=e.index + 37 * (l + 1))))
    for l, lw in enumerate(w["dec_layers"]):
        lw.update(make_random_scales(replace(d, index=d.index + 37 * (l + 1))))
    rng = np.random.default_rng(BASE_SEED + 1000 * e.index + 504)
    w["enc_final_scale"] = round_to_dtype(1.0 + 0.1 * rng.standard_normal(e.d_model), e.dtype)
    w["dec_final_scale"] = round_to_dtype(1.0 + 0.1 * rng.standard_normal(d.d_model), d.dtype)


def make_encdec_tokens(ec: EncDecConfig, seed_offset: int = 0, ignore_fraction: float = 0.1) -> tuple:
    """(enc_tokens [B, S_enc], dec_tokens [B, S_dec], targets [B, S_dec]) int32, Zipf-like as make_tokens."""
    enc_tokens, _ = make_tokens(StackConfig("e", ec.enc_block, 1, ec.vocab), seed_offset, 0.0)
    dec_tokens, targets = make_tokens(StackConfig("d", ec.dec_block, 1, ec.vocab), seed_offset, ignore_fraction)
    return enc_tokens, dec_tokens, targets


def make_adafactor_case(rows: int, cols: int, seed: int, grad_std: float = 1e-2) -> tuple:
    """(param, grad) float64 arrays holding float32-representable values for a standalone optimizer test."""
    rng = np.random.default_rng(BASE_SEED + 7919 * seed + rows * 31 + cols)
    p = rng.standard_normal((rows, cols)) * (max(rows, 1) ** -0.5)
    g = rng.standard_normal((rows, cols)) * grad_std
    # column- and row-dependent gradient scale so the factored statistics are not flat
    g = g * (0.5 + rng.random((rows, 1))) * (0.5 + rng.random((1, cols)))
    return p.astype(np.float32).astype(np.float64), g.astype(np.float32).astype(np.float64)
