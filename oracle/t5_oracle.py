"""CPU oracle (float64, numpy) for one T5.1.1-style Transformer block and Adafactor.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the HIP
path is checked against.  It shares no code with the HIP path, imports nothing
from it, and may be imported only by tests, the smoke check and the bench's
CPU-baseline leg.  It is never a fallback for the product path.

What it follows.  The paper (Sec. 4, "Example models") ships "T5.1.1" and a
decoder-only configuration as its models and Sec. 2.3 says they are ordinary
Flax modules, but it prints no formula for any layer.  Every formula below is
therefore the public definition of the named layer, written out in full:

  * T5 layer norm: scale-only RMS norm, no mean subtraction, no bias.
  * Self-attention whose logits get a learned bias looked up from a table by
    the *bucket* of (key position - query position); no 1/sqrt(d_kv) factor
    unless the caller asks for one through attn_scale.
  * T5.1.1 feed-forward: gated GELU (tanh form), no biases.  Variants: the exact (erf)
    GELU in the same gated form, and the original T5's ungated ReLU feed-forward.
  * Pre-norm residual wiring: h = x + Attn(Norm(x)); y = h + MLP(Norm(h)).
  * Stack: token embedding (no input scaling), N blocks sharing one relative-position
    table, final RMSNorm, logits (untied output matrix, or the embedding transposed
    and scaled by d_model^-1/2), softmax cross-entropy plus z_loss * log(Z)^2, mean
    over the positions whose target is >= 0.
  * Decoder block of the encoder-decoder model: the same, with a cross-attention
    sublayer (queries from the decoder stream, keys and values from the encoder
    output, no position bias, no mask) between self-attention and the MLP.
  * Adafactor with factored second moments and update clipping, no momentum.

The result has a plain definition, so the oracle *is* that definition: the
S x S score matrix is materialised, softmax is the ordinary two-pass form, and
the backward pass is the hand-derived chain rule written term by term.  The
only library primitive used as a step is numpy's matmul.

All functions take and return float64 arrays.
"""
from __future__ import annotations

import dataclasses
import math
import numpy as np

GELU_KAPPA = math.sqrt(2.0 / math.pi)
GELU_BETA = 0.044715


# --------------------------------------------------------------------------------------
# Relative-position buckets (integer, exact)
# --------------------------------------------------------------------------------------
def relpos_bucket_scalar(rel_pos: int, bidirectional: bool, num_buckets: int = 32,
                         max_distance: int = 128) -> int:
    """Bucket of one relative position rel_pos = key_position - query_position.

    T5 definition.  Half of the buckets (per sign when bidirectional) are exact
    offsets; the other half are logarithmically spaced up to max_distance, and
    everything beyond shares the last bucket.  In unidirectional (causal) mode
    only keys at or before the query are distinguished; keys after the query
    collapse to bucket 0 (they are masked anyway).

    The logarithmic part is floor(L * ln(n/E) / ln(D/E)) with E the number of
    exact buckets, L the number of logarithmic ones and D = max_distance.  It
    is evaluated here in exact integer arithmetic: the floor is the largest K
    with (n/E)^L >= (D/E)^K, i.e. n^L * E^K >= D^K * E^L.  Python integers are
    unbounded, so no rounding can move a boundary.
    """
    rp = int(rel_pos)
    n_side = num_buckets
    base = 0
    if bidirectional:
        n_side = num_buckets // 2
        if rp > 0:
            base = n_side
        n = abs(rp)
    else:
        n = max(-rp, 0)
    max_exact = n_side // 2
    if n < max_exact:
        return base + n
    n_log = n_side - max_exact
    big_k = 0
    # largest K with n^L * E^K >= D^K * E^L ; K can not usefully exceed n_log
    while big_k + 1 <= n_log and (n ** n_log) * (max_exact ** (big_k + 1)) >= \
            (max_distance ** (big_k + 1)) * (max_exact ** n_log):
        big_k += 1
    return base + min(n_side - 1, max_exact + big_k)


def relpos_bucket(rel_pos, bidirectional: bool, num_buckets: int = 32, max_distance: int = 128):
    """Vectorised wrapper of relpos_bucket_scalar; returns int64 array of the input's shape."""
    rp = np.asarray(rel_pos)
    out = np.empty(rp.shape, dtype=np.int64)
    flat_in, flat_out = rp.reshape(-1), out.reshape(-1)
    cache = {}
    for idx in range(flat_in.size):
        v = int(flat_in[idx])
        if v not in cache:
            cache[v] = relpos_bucket_scalar(v, bidirectional, num_buckets, max_distance)
        flat_out[idx] = cache[v]
    return out


def relpos_bias(rel_table: np.ndarray, seq: int, bidirectional: bool, num_buckets: int,
                max_distance: int) -> np.ndarray:
    """bias[h, i, j] = rel_table[bucket(j - i), h]   (query i, key j)."""
    pos = np.arange(seq)
    rp = pos[None, :] - pos[:, None]          # rp[i, j] = j - i
    bucket = relpos_bucket(rp, bidirectional, num_buckets, max_distance)
    return np.transpose(rel_table[bucket], (2, 0, 1)), bucket


# --------------------------------------------------------------------------------------
# Layer pieces
# --------------------------------------------------------------------------------------
def rmsnorm_fwd(x: np.ndarray, g: np.ndarray, eps: float):
    """n = x * r * g with r = (mean_c x_c^2 + eps)^-1/2 taken over the last axis."""
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return x * r * g, r


def rmsnorm_bwd(x: np.ndarray, g: np.ndarray, r: np.ndarray, dn: np.ndarray):
    """Gradient of rmsnorm_fwd.  With xh = x r:  dg = sum_tokens dn*xh,
    dxh = dn*g,  dx = r * (dxh - xh * mean_c(dxh*xh))."""
    xh = x * r
    dg = np.sum((dn * xh).reshape(-1, x.shape[-1]), axis=0)
    dxh = dn * g
    dx = r * (dxh - xh * np.mean(dxh * xh, axis=-1, keepdims=True))
    return dx, dg


def gelu(z: np.ndarray) -> np.ndarray:
    """tanh-form GELU: z/2 * (1 + tanh(kappa (z + beta z^3)))."""
    return 0.5 * z * (1.0 + np.tanh(GELU_KAPPA * (z + GELU_BETA * z ** 3)))


def gelu_grad(z: np.ndarray) -> np.ndarray:
    t = np.tanh(GELU_KAPPA * (z + GELU_BETA * z ** 3))
    return 0.5 * (1.0 + t) + 0.5 * z * (1.0 - t * t) * GELU_KAPPA * (1.0 + 3.0 * GELU_BETA * z * z)


def gelu_erf(z: np.ndarray) -> np.ndarray:
    """Exact GELU: z * Phi(z), Phi the standard normal distribution function."""
    erf = np.vectorize(math.erf, otypes=[np.float64])
    return 0.5 * z * (1.0 + erf(z / math.sqrt(2.0)))


def gelu_erf_grad(z: np.ndarray) -> np.ndarray:
    erf = np.vectorize(math.erf, otypes=[np.float64])
    return 0.5 * (1.0 + erf(z / math.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)


def mlp_fwd(cfg, n2: np.ndarray, w: dict, hidden_scale=None):
    """Feed-forward sublayer without its norm and residual, by cfg.mlp:
      "geglu_tanh" (T5.1.1): a = gelu_tanh(n2 Wi0) * (n2 Wi1)
      "geglu_erf":           the same with the exact GELU
      "relu" (original T5):  a = max(n2 Wi0, 0), no gate and no Wi1
    hidden_scale (dropout on the hidden activation, or None) multiplies a before the output projection.
    Returns (a Wo_ff, saved); saved["a"] is the activation the output projection saw."""
    kind = getattr(cfg, "mlp", "geglu_tanh")
    u = n2 @ w["wi0"]
    if kind == "relu":
        a = np.maximum(u, 0.0)
        if hidden_scale is not None:
            a = a * hidden_scale
        return a @ w["wo_ff"], dict(u=u, a=a)
    act = gelu if kind == "geglu_tanh" else gelu_erf
    wl = n2 @ w["wi1"]
    a = act(u) * wl
    if hidden_scale is not None:
        a = a * hidden_scale
    return a @ w["wo_ff"], dict(u=u, wl=wl, a=a)


def mlp_bwd(cfg, dout: np.ndarray, n2: np.ndarray, w: dict, sv: dict, hidden_scale=None):
    """Given dout = gradient of the sublayer's output: (dn2, {wo_ff, wi0[, wi1]} gradients)."""
    kind = getattr(cfg, "mlp", "geglu_tanh")
    flat = lambda t: t.reshape(-1, t.shape[-1])
    g = {"wo_ff": flat(sv["a"]).T @ flat(dout)}
    da = dout @ w["wo_ff"].T
    if hidden_scale is not None:
        da = da * hidden_scale
    if kind == "relu":
        du = da * (sv["u"] > 0.0)
        g["wi0"] = flat(n2).T @ flat(du)
        return du @ w["wi0"].T, g
    act, act_grad = (gelu, gelu_grad) if kind == "geglu_tanh" else (gelu_erf, gelu_erf_grad)
    du = da * sv["wl"] * act_grad(sv["u"])
    dwl = da * act(sv["u"])
    g["wi0"] = flat(n2).T @ flat(du)
    g["wi1"] = flat(n2).T @ flat(dwl)
    return du @ w["wi0"].T + dwl @ w["wi1"].T, g


def softmax_rows(s: np.ndarray) -> np.ndarray:
    """Two-pass softmax over the last axis; -inf entries get probability exactly 0."""
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


# --------------------------------------------------------------------------------------
# Dropout with a counter-based generator
# --------------------------------------------------------------------------------------
# Sites of a block, as in the T5 models (paper Sec. 4): attention probabilities, the attention sublayer's
# output, the feed-forward hidden activation and the feed-forward sublayer's output.
DROP_ATTN_PROBS, DROP_ATTN_OUT, DROP_MLP_HIDDEN, DROP_MLP_OUT = 1, 2, 3, 4
# the cross-attention sublayer of a decoder layer, and the two ends of a stack (embedded tokens; output of the
# final norm); the decoder side of an encoder-decoder pair has its own end sites
DROP_CROSS_PROBS, DROP_CROSS_OUT, DROP_EMBED, DROP_FINAL, DROP_DEC_EMBED, DROP_DEC_FINAL = 5, 6, 7, 8, 9, 10


def _mix32(x: np.ndarray) -> np.ndarray:
    """A 32-bit integer finaliser (xor-shift / odd-multiply rounds, the public-domain 'lowbias32'
    constants) on uint64 arrays holding 32-bit values; every step is reduced mod 2^32."""
    m = np.uint64(0xFFFFFFFF)
    x = x & m
    x = x ^ (x >> np.uint64(16))
    x = (x * np.uint64(0x7FEB352D)) & m
    x = x ^ (x >> np.uint64(15))
    x = (x * np.uint64(0x846CA68B)) & m
    x = x ^ (x >> np.uint64(16))
    return x


def dropout_keep(seed: int, site: int, n_hi: int, n_lo: int, rate: float) -> np.ndarray:
    """Boolean keep mask [n_hi, n_lo] of a dropout site.  Element (hi, lo) is a pure function of
    (seed, site, hi, lo) -- no state, so the forward, the backward and any tiling regenerate it:
        k0 = mix32(seed_lo ^ (site * 0x9E3779B9 mod 2^32))
        k1 = mix32(k0 ^ hi ^ seed_hi)            one per row
        r  = mix32(k1 ^ lo)                      one per element
        keep = r >= floor(rate * 2^32)
    hi is the row (token, or (batch*heads + head)*seq + query for attention probabilities), lo the column
    (channel, hidden unit, or key position)."""
    m = np.uint64(0xFFFFFFFF)
    seed_lo, seed_hi = np.uint64(seed & 0xFFFFFFFF), np.uint64((seed >> 32) & 0xFFFFFFFF)
    k0 = _mix32(np.array([seed_lo ^ np.uint64((site * 0x9E3779B9) & 0xFFFFFFFF)], dtype=np.uint64))[0]
    hi = np.arange(n_hi, dtype=np.uint64)[:, None]
    lo = np.arange(n_lo, dtype=np.uint64)[None, :]
    k1 = _mix32(k0 ^ hi ^ seed_hi)
    r = _mix32(k1 ^ lo)
    thr = np.uint64(min(int(math.floor(rate * 4294967296.0)), 0xFFFFFFFF))
    return r >= thr


def dropout_layer_seed(seed: int, layer: int) -> int:
    """Seed of layer `layer` (0-based) of a stack whose configuration carries `seed`: the layers must not
    share masks, so each adds a multiple of an odd 64-bit constant (mod 2^64).  The decoder layers of an
    encoder-decoder pair count on from the encoder's."""
    return (seed + (layer + 1) * 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF


def _with_layer_seed(cfg, layer: int):
    if getattr(cfg, "dropout_rate", 0.0) <= 0.0:
        return cfg
    return dataclasses.replace(cfg, dropout_seed=dropout_layer_seed(cfg.dropout_seed, layer))


def _token_scale(cfg, site: int, shape):
    """Multiplier of a per-token site for activations of shape [B, S, width]; 1.0 when dropout is off."""
    m = dropout_scale(cfg, site, shape[0] * shape[1], shape[2])
    return 1.0 if m is None else m.reshape(shape)


def dropout_scale(cfg, site: int, n_hi: int, n_lo: int):
    """Multiplier of a site: 1 / (1 - rate) where kept, 0 where dropped; None when dropout is off."""
    rate = getattr(cfg, "dropout_rate", 0.0)
    if rate <= 0.0:
        return None
    return dropout_keep(cfg.dropout_seed, site, n_hi, n_lo, rate) / (1.0 - rate)


# --------------------------------------------------------------------------------------
# Block forward / backward
# --------------------------------------------------------------------------------------
def _split_heads(t: np.ndarray, n_heads: int, d_kv: int) -> np.ndarray:
    b, s, _ = t.shape                          # [B,S,H*k] -> [B,H,S,k]; column h*k+c = head h, channel c
    return np.transpose(t.reshape(b, s, n_heads, d_kv), (0, 2, 1, 3))


def _merge_heads(t: np.ndarray) -> np.ndarray:
    b, h, s, k = t.shape
    return np.transpose(t, (0, 2, 1, 3)).reshape(b, s, h * k)


def block_fwd(cfg, x: np.ndarray, w: dict):
    """y = block(x).  x: [B,S,d].  Returns (y, saved) with every intermediate kept for the backward.

    Steps (one sequence at a time is implied by the batched matmuls):
      n1 = RMSNorm(x; g1);  q,k,v = n1 Wq, n1 Wk, n1 Wv  (split into heads)
      s[h,i,j] = attn_scale <q_hi, k_hj> + table[bucket(j-i), h];  causal: j>i -> -inf
      P = softmax_j s;  o = P v;  c = concat_h o;  h = x + c Wo
      n2 = RMSNorm(h; g2);  u = n2 Wi0;  w = n2 Wi1;  a = gelu(u) * w;  y = h + a Wo_ff
    """
    nh, dk = cfg.n_heads, cfg.d_kv
    n1, r1 = rmsnorm_fwd(x, w["ln1_scale"], cfg.rms_eps)
    q = _split_heads(n1 @ w["wq"], nh, dk)
    k = _split_heads(n1 @ w["wk"], nh, dk)
    v = _split_heads(n1 @ w["wv"], nh, dk)
    bias, bucket = relpos_bias(w["rel_table"], cfg.seq, not cfg.causal, cfg.num_buckets, cfg.max_distance)
    s = cfg.attn_scale * (q @ np.swapaxes(k, -1, -2)) + bias[None]
    if cfg.causal:
        i = np.arange(cfg.seq)
        s = np.where(i[None, :] > i[:, None], -np.inf, s)
    p = softmax_rows(s)
    # dropout (training only; cfg.dropout_rate = 0 leaves every site untouched)
    B, S = x.shape[0], cfg.seq
    drop = {site: dropout_scale(cfg, site, n_hi, n_lo) for site, n_hi, n_lo in
            ((DROP_ATTN_PROBS, B * nh * S, S), (DROP_ATTN_OUT, B * S, cfg.d_model),
             (DROP_MLP_HIDDEN, B * S, cfg.d_ff), (DROP_MLP_OUT, B * S, cfg.d_model))}
    if drop[DROP_ATTN_PROBS] is not None:
        drop = {DROP_ATTN_PROBS: drop[DROP_ATTN_PROBS].reshape(B, nh, S, S),
                DROP_ATTN_OUT: drop[DROP_ATTN_OUT].reshape(B, S, -1),
                DROP_MLP_HIDDEN: drop[DROP_MLP_HIDDEN].reshape(B, S, -1),
                DROP_MLP_OUT: drop[DROP_MLP_OUT].reshape(B, S, -1)}
    on = drop[DROP_ATTN_PROBS] is not None
    pd = p * drop[DROP_ATTN_PROBS] if on else p          # what multiplies v
    o = pd @ v
    c = _merge_heads(o)
    ao = c @ w["wo"]
    h = x + (ao * drop[DROP_ATTN_OUT] if on else ao)
    n2, r2 = rmsnorm_fwd(h, w["ln2_scale"], cfg.rms_eps)
    mlp_out, mlp_saved = mlp_fwd(cfg, n2, w, drop[DROP_MLP_HIDDEN])
    y = h + (mlp_out * drop[DROP_MLP_OUT] if on else mlp_out)
    saved = dict(x=x, n1=n1, r1=r1, q=q, k=k, v=v, p=p, pd=pd, c=c, h=h, n2=n2, r2=r2, bucket=bucket,
                 drop=drop if on else None, **mlp_saved)
    return y, saved


def block_bwd(cfg, dy: np.ndarray, w: dict, saved: dict):
    """Gradients of sum(y * dy) w.r.t. x and every weight.  Returns (dx, grads)."""
    nh, dk = cfg.n_heads, cfg.d_kv
    d = cfg.d_model
    x, n1, r1, q, k, v, p, c, h, n2, r2 = (saved[t] for t in
        ("x", "n1", "r1", "q", "k", "v", "p", "c", "h", "n2", "r2"))
    flat = lambda t: t.reshape(-1, t.shape[-1])
    drop = saved.get("drop")
    # --- MLP
    dout = dy * drop[DROP_MLP_OUT] if drop else dy
    dn2, g = mlp_bwd(cfg, dout, n2, w, saved, drop[DROP_MLP_HIDDEN] if drop else None)
    dh_norm, g["ln2_scale"] = rmsnorm_bwd(h, w["ln2_scale"], r2, dn2)
    dh = dy + dh_norm
    # --- attention
    dao = dh * drop[DROP_ATTN_OUT] if drop else dh
    g["wo"] = flat(c).T @ flat(dao)
    dc = dao @ w["wo"].T
    do = _split_heads(dc, nh, dk)
    dv = np.swapaxes(saved["pd"], -1, -2) @ do
    dp = do @ np.swapaxes(v, -1, -2)
    if drop:
        dp = dp * drop[DROP_ATTN_PROBS]
    ds = p * (dp - np.sum(p * dp, axis=-1, keepdims=True))      # masked entries have p = 0 -> ds = 0
    dq = cfg.attn_scale * (ds @ k)
    dk_ = cfg.attn_scale * (np.swapaxes(ds, -1, -2) @ q)
    # bias table: every (b, i, j) adds ds[b,h,i,j] to row bucket(j-i) of column h
    dtable = np.zeros_like(w["rel_table"])
    ds_hij = np.sum(ds, axis=0)                                 # [H,S,S]
    for hh in range(nh):
        np.add.at(dtable[:, hh], saved["bucket"].reshape(-1), ds_hij[hh].reshape(-1))
    g["rel_table"] = dtable
    dqf, dkf, dvf = _merge_heads(dq), _merge_heads(dk_), _merge_heads(dv)
    g["wq"] = flat(n1).T @ flat(dqf)
    g["wk"] = flat(n1).T @ flat(dkf)
    g["wv"] = flat(n1).T @ flat(dvf)
    dn1 = dqf @ w["wq"].T + dkf @ w["wk"].T + dvf @ w["wv"].T
    dx_norm, g["ln1_scale"] = rmsnorm_bwd(x, w["ln1_scale"], r1, dn1)
    dx = dh + dx_norm
    assert dx.shape[-1] == d
    return dx, g


# --------------------------------------------------------------------------------------
# Decoder block: causal self-attention, cross-attention over an encoder output, MLP
# --------------------------------------------------------------------------------------
def decoder_block_fwd(cfg, x: np.ndarray, enc: np.ndarray, w: dict):
    """y = decoder_block(x, enc).  x: [B,S,d] decoder stream, enc: [B,S_enc,d] encoder output.

    The encoder-decoder T5 of the paper (Sec. 4) stacks this layer in its decoder.  Pre-norm
    residual wiring with three sublayers:
      h1 = x  + SelfAttn(RMSNorm(x; g1))                 (as in block_fwd: bias table, causal mask)
      h2 = h1 + CrossAttn(RMSNorm(h1; gx), enc)
      y  = h2 + MLP(RMSNorm(h2; g2))
    Cross-attention: queries from the normalised decoder stream, keys and values from the encoder
    output as it is (it was normalised by the encoder's final norm); no position bias, no mask:
      q = nx Xq;  k = enc Xk;  v = enc Xv  (split into heads)
      s[h,i,j] = attn_scale <q_hi, k_hj>;  P = softmax_j s;  o = P v;  cx = concat_h o;  h2 = h1 + cx Xo
    """
    nh, dk = cfg.n_heads, cfg.d_kv
    # --- self-attention sublayer
    n1, r1 = rmsnorm_fwd(x, w["ln1_scale"], cfg.rms_eps)
    q = _split_heads(n1 @ w["wq"], nh, dk)
    k = _split_heads(n1 @ w["wk"], nh, dk)
    v = _split_heads(n1 @ w["wv"], nh, dk)
    bias, bucket = relpos_bias(w["rel_table"], cfg.seq, not cfg.causal, cfg.num_buckets, cfg.max_distance)
    s = cfg.attn_scale * (q @ np.swapaxes(k, -1, -2)) + bias[None]
    if cfg.causal:
        i = np.arange(cfg.seq)
        s = np.where(i[None, :] > i[:, None], -np.inf, s)
    p = softmax_rows(s)
    # dropout: the block's four sites plus the two of the cross-attention sublayer (rows of its probabilities:
    # (b*H + h)*S + i over the S decoder positions, columns: encoder positions)
    B, S, Se = x.shape[0], cfg.seq, enc.shape[1]
    drop = None
    if getattr(cfg, "dropout_rate", 0.0) > 0.0:
        drop = {DROP_ATTN_PROBS: dropout_scale(cfg, DROP_ATTN_PROBS, B * nh * S, S).reshape(B, nh, S, S),
                DROP_ATTN_OUT: dropout_scale(cfg, DROP_ATTN_OUT, B * S, cfg.d_model).reshape(B, S, -1),
                DROP_CROSS_PROBS: dropout_scale(cfg, DROP_CROSS_PROBS, B * nh * S, Se).reshape(B, nh, S, Se),
                DROP_CROSS_OUT: dropout_scale(cfg, DROP_CROSS_OUT, B * S, cfg.d_model).reshape(B, S, -1),
                DROP_MLP_HIDDEN: dropout_scale(cfg, DROP_MLP_HIDDEN, B * S, cfg.d_ff).reshape(B, S, -1),
                DROP_MLP_OUT: dropout_scale(cfg, DROP_MLP_OUT, B * S, cfg.d_model).reshape(B, S, -1)}
    one = lambda site: drop[site] if drop else 1.0
    pd = p * one(DROP_ATTN_PROBS)
    c = _merge_heads(pd @ v)
    h1 = x + (c @ w["wo"]) * one(DROP_ATTN_OUT)
    # --- cross-attention sublayer
    nx, rx = rmsnorm_fwd(h1, w["lnx_scale"], cfg.rms_eps)
    qx = _split_heads(nx @ w["xq"], nh, dk)
    kx = _split_heads(enc @ w["xk"], nh, dk)
    vx = _split_heads(enc @ w["xv"], nh, dk)
    px = softmax_rows(cfg.attn_scale * (qx @ np.swapaxes(kx, -1, -2)))
    pxd = px * one(DROP_CROSS_PROBS)
    cx = _merge_heads(pxd @ vx)
    h2 = h1 + (cx @ w["xo"]) * one(DROP_CROSS_OUT)
    # --- MLP sublayer
    n2, r2 = rmsnorm_fwd(h2, w["ln2_scale"], cfg.rms_eps)
    mlp_out, mlp_saved = mlp_fwd(cfg, n2, w, drop[DROP_MLP_HIDDEN] if drop else None)
    y = h2 + mlp_out * one(DROP_MLP_OUT)
    saved = dict(x=x, enc=enc, n1=n1, r1=r1, q=q, k=k, v=v, p=p, pd=pd, c=c, h1=h1, nx=nx, rx=rx, qx=qx, kx=kx,
                 vx=vx, px=px, pxd=pxd, cx=cx, h2=h2, n2=n2, r2=r2, bucket=bucket, drop=drop, **mlp_saved)
    return y, saved


def decoder_block_bwd(cfg, dy: np.ndarray, w: dict, saved: dict):
    """Gradients of sum(y * dy) w.r.t. x, enc and every weight.  Returns (dx, denc, grads)."""
    nh, dk = cfg.n_heads, cfg.d_kv
    flat = lambda t: t.reshape(-1, t.shape[-1])
    sv = saved
    drop = sv.get("drop")
    one = lambda site: drop[site] if drop else 1.0
    # --- MLP sublayer
    dn2, g = mlp_bwd(cfg, dy * one(DROP_MLP_OUT), sv["n2"], w, sv, drop[DROP_MLP_HIDDEN] if drop else None)
    dh2_norm, g["ln2_scale"] = rmsnorm_bwd(sv["h2"], w["ln2_scale"], sv["r2"], dn2)
    dh2 = dy + dh2_norm
    # --- cross-attention sublayer
    dxo = dh2 * one(DROP_CROSS_OUT)
    g["xo"] = flat(sv["cx"]).T @ flat(dxo)
    dox = _split_heads(dxo @ w["xo"].T, nh, dk)
    px, qx, kx, vx = sv["px"], sv["qx"], sv["kx"], sv["vx"]
    dvx = np.swapaxes(sv["pxd"], -1, -2) @ dox
    dpx = (dox @ np.swapaxes(vx, -1, -2)) * one(DROP_CROSS_PROBS)
    dsx = px * (dpx - np.sum(px * dpx, axis=-1, keepdims=True))
    dqx = _merge_heads(cfg.attn_scale * (dsx @ kx))
    dkx = _merge_heads(cfg.attn_scale * (np.swapaxes(dsx, -1, -2) @ qx))
    dvx = _merge_heads(dvx)
    g["xq"] = flat(sv["nx"]).T @ flat(dqx)
    g["xk"] = flat(sv["enc"]).T @ flat(dkx)
    g["xv"] = flat(sv["enc"]).T @ flat(dvx)
    denc = dkx @ w["xk"].T + dvx @ w["xv"].T
    dh1_norm, g["lnx_scale"] = rmsnorm_bwd(sv["h1"], w["lnx_scale"], sv["rx"], dqx @ w["xq"].T)
    dh1 = dh2 + dh1_norm
    # --- self-attention sublayer
    dao = dh1 * one(DROP_ATTN_OUT)
    g["wo"] = flat(sv["c"]).T @ flat(dao)
    do = _split_heads(dao @ w["wo"].T, nh, dk)
    p, q, k, v = sv["p"], sv["q"], sv["k"], sv["v"]
    dv = np.swapaxes(sv["pd"], -1, -2) @ do
    dp = (do @ np.swapaxes(v, -1, -2)) * one(DROP_ATTN_PROBS)
    ds = p * (dp - np.sum(p * dp, axis=-1, keepdims=True))
    dq = cfg.attn_scale * (ds @ k)
    dk_ = cfg.attn_scale * (np.swapaxes(ds, -1, -2) @ q)
    dtable = np.zeros_like(w["rel_table"])
    ds_hij = np.sum(ds, axis=0)
    for hh in range(nh):
        np.add.at(dtable[:, hh], sv["bucket"].reshape(-1), ds_hij[hh].reshape(-1))
    g["rel_table"] = dtable
    dqf, dkf, dvf = _merge_heads(dq), _merge_heads(dk_), _merge_heads(dv)
    g["wq"] = flat(sv["n1"]).T @ flat(dqf)
    g["wk"] = flat(sv["n1"]).T @ flat(dkf)
    g["wv"] = flat(sv["n1"]).T @ flat(dvf)
    dn1 = dqf @ w["wq"].T + dkf @ w["wk"].T + dvf @ w["wv"].T
    dx_norm, g["ln1_scale"] = rmsnorm_bwd(sv["x"], w["ln1_scale"], sv["r1"], dn1)
    return dh1 + dx_norm, denc, g


# --------------------------------------------------------------------------------------
# Stack of blocks with token embedding, final norm, logits and loss
# --------------------------------------------------------------------------------------
def xent_zloss(logits: np.ndarray, targets: np.ndarray, z_loss: float):
    """Softmax cross-entropy with the auxiliary z-loss of the T5 training recipe, per position:
        lse = log sum_v exp(logits_v);   loss = lse - logits[target] + z_loss * lse^2
    Positions with target < 0 carry no loss.  Returns (mean over the positions that count, lse,
    number of positions that count).  logits: [..., V], targets: integer [...]"""
    m = logits.max(axis=-1, keepdims=True)
    lse = (m + np.log(np.exp(logits - m).sum(axis=-1, keepdims=True)))[..., 0]
    valid = targets >= 0
    picked = np.take_along_axis(logits, np.where(valid, targets, 0)[..., None], axis=-1)[..., 0]
    per = np.where(valid, lse - picked + z_loss * lse * lse, 0.0)
    n = int(valid.sum())
    return float(per.sum() / max(n, 1)), lse, n


def xent_zloss_grad(logits: np.ndarray, targets: np.ndarray, lse: np.ndarray, z_loss: float, n: int):
    """d(mean loss)/d(logits): (softmax * (1 + 2 z_loss lse) - onehot(target)) / n on counted positions."""
    p = np.exp(logits - lse[..., None])
    g = p * (1.0 + 2.0 * z_loss * lse)[..., None]
    valid = targets >= 0
    idx = np.where(valid, targets, 0)[..., None]
    np.put_along_axis(g, idx, np.take_along_axis(g, idx, axis=-1) - 1.0, axis=-1)
    return g * (valid[..., None] / max(n, 1))


def stack_loss(sc, tokens: np.ndarray, targets: np.ndarray, w: dict):
    """Training loss of the stack (paper Sec. 4 models as plain layer stacks, Sec. 2.3):
        x_0 = E[tokens];  x_{l+1} = block_l(x_l)  with ONE relative-position table shared by all layers
        nf = RMSNorm(x_L; gf);  logits = nf Wout   (tied: logits = d_model^-1/2 nf E^T)
        loss = mean over positions with target >= 0 of xent_zloss
    With dropout (block.dropout_rate > 0): layer l runs with the seed dropout_layer_seed(seed, l), the embedded
    tokens pass site DROP_EMBED and the output of the final norm site DROP_FINAL (both under the stack's seed).
    Returns (loss, saved)."""
    cfg = sc.block
    x = w["embedding"][tokens]
    m_embed = _token_scale(cfg, DROP_EMBED, x.shape)
    x = x * m_embed
    saved_layers = []
    for l, lw in enumerate(w["layers"]):
        wl = dict(lw, rel_table=w["rel_table"])
        x, sv = block_fwd(_with_layer_seed(cfg, l), x, wl)
        saved_layers.append(sv)
    nf, rf = rmsnorm_fwd(x, w["final_scale"], cfg.rms_eps)
    m_final = _token_scale(cfg, DROP_FINAL, nf.shape)
    nf = nf * m_final                                    # what the logits see
    if sc.tied_logits:
        logits = (nf * cfg.d_model ** -0.5) @ w["embedding"].T
    else:
        logits = nf @ w["logits_w"]
    loss, lse, n = xent_zloss(logits, targets, sc.z_loss)
    return loss, dict(tokens=tokens, targets=targets, layers=saved_layers, x_last=x, nf=nf, rf=rf, logits=logits,
                      lse=lse, n=n, m_embed=m_embed, m_final=m_final)


def stack_loss_grad(sc, w: dict, saved: dict) -> dict:
    """Gradient of stack_loss w.r.t. every weight: {"embedding", "rel_table" (summed over layers),
    "final_scale", "logits_w" (untied), "layers": [block gradient dicts without rel_table]}."""
    cfg = sc.block
    flat = lambda t: t.reshape(-1, t.shape[-1])
    dlogits = xent_zloss_grad(saved["logits"], saved["targets"], saved["lse"], sc.z_loss, saved["n"])
    g = {"layers": [None] * sc.n_layers, "embedding": np.zeros_like(w["embedding"])}
    if sc.tied_logits:
        s = cfg.d_model ** -0.5
        g["embedding"] += s * (flat(dlogits).T @ flat(saved["nf"]))
        dnf = s * (dlogits @ w["embedding"])
    else:
        g["logits_w"] = flat(saved["nf"]).T @ flat(dlogits)
        dnf = dlogits @ w["logits_w"].T
    dx, g["final_scale"] = rmsnorm_bwd(saved["x_last"], w["final_scale"], saved["rf"], dnf * saved["m_final"])
    g["rel_table"] = np.zeros_like(w["rel_table"])
    for l in range(sc.n_layers - 1, -1, -1):
        wl = dict(w["layers"][l], rel_table=w["rel_table"])
        dx, gl = block_bwd(_with_layer_seed(cfg, l), dx, wl, saved["layers"][l])
        g["rel_table"] += gl.pop("rel_table")
        g["layers"][l] = gl
    np.add.at(g["embedding"], saved["tokens"].reshape(-1), flat(dx * saved["m_embed"]))
    return g


def encdec_loss(ec, enc_tokens: np.ndarray, dec_tokens: np.ndarray, targets: np.ndarray, w: dict):
    """Training loss of the encoder-decoder model (paper Sec. 4, T5.1.1):
        enc_out = RMSNorm(encoder blocks(E[enc_tokens]); enc_final_scale)    bidirectional, own shared table
        x_{l+1} = decoder_block_l(x_l, enc_out),  x_0 = E[dec_tokens]        causal, own shared table
        nf = RMSNorm(x_L; dec_final_scale);  logits, loss as in stack_loss
    With dropout each side takes rate and seed from its own block configuration: encoder layer l runs with
    dropout_layer_seed(seed, l), decoder layer l with dropout_layer_seed(seed, n_enc_layers + l); the encoder's
    ends are sites DROP_EMBED / DROP_FINAL (enc_out is the dropped norm output), the decoder's
    DROP_DEC_EMBED / DROP_DEC_FINAL.
    Returns (loss, saved)."""
    e, d = ec.enc_block, ec.dec_block
    x = w["embedding"][enc_tokens]
    me_embed = _token_scale(e, DROP_EMBED, x.shape)
    x = x * me_embed
    enc_saved = []
    for l, lw in enumerate(w["enc_layers"]):
        x, sv = block_fwd(_with_layer_seed(e, l), x, dict(lw, rel_table=w["enc_rel_table"]))
        enc_saved.append(sv)
    enc_out, enc_rf = rmsnorm_fwd(x, w["enc_final_scale"], e.rms_eps)
    me_final = _token_scale(e, DROP_FINAL, enc_out.shape)
    enc_out = enc_out * me_final
    xe_last = x
    x = w["embedding"][dec_tokens]
    md_embed = _token_scale(d, DROP_DEC_EMBED, x.shape)
    x = x * md_embed
    dec_saved = []
    for l, lw in enumerate(w["dec_layers"]):
        x, sv = decoder_block_fwd(_with_layer_seed(d, ec.n_enc_layers + l), x, enc_out,
                                  dict(lw, rel_table=w["dec_rel_table"]))
        dec_saved.append(sv)
    nf, rf = rmsnorm_fwd(x, w["dec_final_scale"], d.rms_eps)
    md_final = _token_scale(d, DROP_DEC_FINAL, nf.shape)
    nf = nf * md_final
    if ec.tied_logits:
        logits = (nf * d.d_model ** -0.5) @ w["embedding"].T
    else:
        logits = nf @ w["logits_w"]
    loss, lse, n = xent_zloss(logits, targets, ec.z_loss)
    return loss, dict(enc_tokens=enc_tokens, dec_tokens=dec_tokens, targets=targets, enc_layers=enc_saved,
                      dec_layers=dec_saved, xe_last=xe_last, enc_rf=enc_rf, x_last=x, nf=nf, rf=rf, logits=logits,
                      lse=lse, n=n, masks=(me_embed, me_final, md_embed, md_final))


def encdec_loss_grad(ec, w: dict, saved: dict) -> dict:
    """Gradient of encdec_loss w.r.t. every weight (same nesting as the weights)."""
    e, d = ec.enc_block, ec.dec_block
    flat = lambda t: t.reshape(-1, t.shape[-1])
    dlogits = xent_zloss_grad(saved["logits"], saved["targets"], saved["lse"], ec.z_loss, saved["n"])
    g = {"embedding": np.zeros_like(w["embedding"]), "enc_layers": [None] * ec.n_enc_layers,
         "dec_layers": [None] * ec.n_dec_layers}
    if ec.tied_logits:
        s = d.d_model ** -0.5
        g["embedding"] += s * (flat(dlogits).T @ flat(saved["nf"]))
        dnf = s * (dlogits @ w["embedding"])
    else:
        g["logits_w"] = flat(saved["nf"]).T @ flat(dlogits)
        dnf = dlogits @ w["logits_w"].T
    me_embed, me_final, md_embed, md_final = saved["masks"]
    dx, g["dec_final_scale"] = rmsnorm_bwd(saved["x_last"], w["dec_final_scale"], saved["rf"], dnf * md_final)
    g["dec_rel_table"] = np.zeros_like(w["dec_rel_table"])
    denc_out = 0.0
    for l in range(ec.n_dec_layers - 1, -1, -1):
        wl = dict(w["dec_layers"][l], rel_table=w["dec_rel_table"])
        dx, denc_l, gl = decoder_block_bwd(_with_layer_seed(d, ec.n_enc_layers + l), dx, wl, saved["dec_layers"][l])
        denc_out = denc_out + denc_l
        g["dec_rel_table"] += gl.pop("rel_table")
        g["dec_layers"][l] = gl
    np.add.at(g["embedding"], saved["dec_tokens"].reshape(-1), flat(dx * md_embed))
    dx, g["enc_final_scale"] = rmsnorm_bwd(saved["xe_last"], w["enc_final_scale"], saved["enc_rf"],
                                           denc_out * me_final)
    g["enc_rel_table"] = np.zeros_like(w["enc_rel_table"])
    for l in range(ec.n_enc_layers - 1, -1, -1):
        wl = dict(w["enc_layers"][l], rel_table=w["enc_rel_table"])
        dx, gl = block_bwd(_with_layer_seed(e, l), dx, wl, saved["enc_layers"][l])
        g["enc_rel_table"] += gl.pop("rel_table")
        g["enc_layers"][l] = gl
    np.add.at(g["embedding"], saved["enc_tokens"].reshape(-1), flat(dx * me_embed))
    return g


# --------------------------------------------------------------------------------------
# Adafactor
# --------------------------------------------------------------------------------------
def adafactor_beta2(step: int, decay_pow: float) -> float:
    """Second-moment decay at 1-based step t: 1 - t^-decay_pow (0 at t = 1)."""
    return 1.0 - float(step) ** (-decay_pow)


def adafactor_step(param: np.ndarray, grad: np.ndarray, state: dict, *, step: int, lr: float,
                   factored: bool, decay_pow: float = 0.8, eps1: float = 1e-30, eps2: float = 1e-3,
                   clip: float = 1.0, scale_by_param: bool = True, beta1: float = 0.0, weight_decay: float = 0.0):
    """One Adafactor update of a [R,C] tensor.  state holds 'vr' [R] and 'vc' [C] when factored,
    else 'v' [R,C], and 'm' [R,C] when beta1 > 0.  Returns (new_param, new_state); inputs are not modified.

      beta2 = 1 - t^-decay_pow
      Q = G*G + eps1
      factored:   vr <- beta2 vr + (1-beta2) mean_j Q;  vc <- beta2 vc + (1-beta2) mean_i Q
                  vhat_ij = vr_i vc_j / mean_i vr_i
      otherwise:  v <- beta2 v + (1-beta2) Q;  vhat = v
      U = G / sqrt(vhat);  U <- U / max(1, RMS(U)/clip)
      alpha = lr * max(eps2, RMS(W))  (or lr alone);  D = alpha U
      beta1 > 0:  m <- beta1 m + (1 - beta1) D;  D = m                 (momentum on the scaled update)
      W <- W - D - lr * weight_decay * W                                (decoupled weight decay)
    """
    b2 = adafactor_beta2(step, decay_pow)
    qm = grad * grad + eps1
    new_state = {}
    if factored:
        vr = b2 * state["vr"] + (1.0 - b2) * np.mean(qm, axis=1)
        vc = b2 * state["vc"] + (1.0 - b2) * np.mean(qm, axis=0)
        vhat = np.outer(vr, vc) / np.mean(vr)
        new_state["vr"], new_state["vc"] = vr, vc
    else:
        vfull = b2 * state["v"] + (1.0 - b2) * qm
        vhat = vfull
        new_state["v"] = vfull
    upd = grad / np.sqrt(vhat)
    rms_u = math.sqrt(float(np.mean(upd * upd)))
    upd = upd / max(1.0, rms_u / clip)
    alpha = lr
    if scale_by_param:
        alpha = lr * max(eps2, math.sqrt(float(np.mean(param * param))))
    delta = alpha * upd
    if beta1 > 0.0:
        new_state["m"] = beta1 * state["m"] + (1.0 - beta1) * delta
        delta = new_state["m"]
    return param - delta - lr * weight_decay * param, new_state


def adafactor_zero_state(rows: int, cols: int, factored: bool, momentum: bool = False) -> dict:
    st = {"vr": np.zeros(rows), "vc": np.zeros(cols)} if factored else {"v": np.zeros((rows, cols))}
    if momentum:
        st["m"] = np.zeros((rows, cols))
    return st
