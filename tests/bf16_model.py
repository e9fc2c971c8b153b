"""Model of the error that bf16 matrix-unit operands alone put into the block's results.

The HIP path multiplies bf16 operands and accumulates in float32; everything between two
contractions (norm statistics, softmax, the residual stream, the activation function, every
weight gradient) is float32.  This module evaluates the forward and backward of a block (and of a
decoder layer with cross-attention) with the oracle's own pieces in float64 and rounds to bf16
(round to nearest even, once) exactly the tensors that reach a matrix unit or are stored in bf16
on the device:

  forward   n1, q, k, v, the unnormalised probabilities exp(s - max) as they enter P V, the
            attention output c, n2, the saved gated-activation factors gp = w act'(u), gl = act(u)
            and a = act(u) w (each formed from the unrounded u, w), and y; in a decoder layer also
            nx, the cross-attention q, k, v, probabilities and output
  backward  du = da gp and dw = da gl, the bf16 copy of the residual-stream gradient that feeds
            an output projection's two gradient GEMMs, dc, the probabilities P as they enter
            dV = P^T dO, ds as it enters dq and dk, dq, dk, dv, dx (and denc)

Everything else stays float64: the residual stream h and its gradient, dn1, dn2, the logits, the
softmax normaliser, the row sums of dO * O, the bias-table gradient and all weight gradients.  No
float32 accumulation error, no reordering, no fast exp: what comes out is the error floor of *ideal*
bf16-operand arithmetic.  The GPU tolerances of the parity tests are derived from this floor
(tests/parity_util.py).

Test infrastructure only; uses numpy, the oracle's layer pieces and the bf16 rounding of the
seeded-input module.
"""
from __future__ import annotations

import numpy as np

import synth_inputs as SI
from oracle import t5_oracle as O


def rb(a: np.ndarray) -> np.ndarray:
    """Round to the nearest bf16 value, returned as float64."""
    return SI.round_to_bf16(a).astype(np.float64)


def _heads(t, nh, dk):      # [B,S,H*k] -> [B,H,S,k]
    b, s, _ = t.shape
    return np.transpose(t.reshape(b, s, nh, dk), (0, 2, 1, 3))


def _merge(t):              # [B,H,S,k] -> [B,S,H*k]
    b, h, s, k = t.shape
    return np.transpose(t, (0, 2, 1, 3)).reshape(b, s, h * k)


def _flat(t):
    return t.reshape(-1, t.shape[-1])


def _act(cfg, u):
    """(act(u), act'(u)) of the gated feed-forward's activation."""
    if cfg.mlp == "geglu_erf":
        return O.gelu_erf(u), O.gelu_erf_grad(u)
    return O.gelu(u), O.gelu_grad(u)


def _keep(cfg, site, shape):
    """Dropout multiplier of a site with [.., rows.., cols] = shape, or None when dropout is off."""
    n_lo = shape[-1]
    n_hi = int(np.prod(shape[:-1]))
    m = O.dropout_scale(cfg, site, n_hi, n_lo)
    return None if m is None else m.reshape(shape)


def _mul(t, m):
    return t if m is None else t * m


def _scores(cfg, q, k, bias, causal):
    s = cfg.attn_scale * (q @ np.swapaxes(k, -1, -2))
    if bias is not None:
        s = s + bias[None]
    if causal:
        i = np.arange(s.shape[-2])
        j = np.arange(s.shape[-1])
        s = np.where(j[None, :] > i[:, None], -np.inf, s)
    m = s.max(-1, keepdims=True)
    e = np.exp(s - m)
    return e, e.sum(-1, keepdims=True)   # the normaliser is that of the undropped, unrounded probabilities


def attention_fwd(cfg, q, k, v, bias, causal, keep):
    """c [B,H,S,k], rounded.  q, k as they enter the score product (bf16, or unrounded in the
    split-operand variants); v bf16."""
    e, l = _scores(cfg, q, k, bias, causal)
    return rb((rb(_mul(e, keep)) @ v) / l)


def attention_bwd(cfg, q, k, v, bias, causal, keep, c, do, q_lp=None, k_lp=None):
    """(dq, dk, dv) rounded and ds unrounded (for the bias-table gradient).  do: gradient of c, bf16.
    q_lp, k_lp: the plain bf16 copies read by the dk and dq contractions when q, k are unrounded."""
    e, l = _scores(cfg, q, k, bias, causal)
    p = e / l
    dvec = np.sum(do * c, -1, keepdims=True)
    dv = rb(np.swapaxes(rb(_mul(p, keep)), -1, -2) @ do)
    ds = p * (_mul(do @ np.swapaxes(v, -1, -2), keep) - dvec)
    dsr = rb(ds)
    dq = rb(cfg.attn_scale * (dsr @ (k if k_lp is None else k_lp)))
    dk = rb(cfg.attn_scale * (np.swapaxes(dsr, -1, -2) @ (q if q_lp is None else q_lp)))
    return dq, dk, dv, ds


# ------------------------------------------------------------------------------ sublayers
def self_attn_fwd(cfg, x, w, split_qk=False, split_n1=False):
    """h = x + SelfAttn(RMSNorm(x)) with h unrounded (the device keeps it in float32).
    split_qk: q and k keep about 16 mantissa bits inside the score product (a two-term bf16 split);
    split_n1: so does n1 inside the q and k projections."""
    nh, dk, S = cfg.n_heads, cfg.d_kv, cfg.seq
    B = x.shape[0]
    n1_full, r1 = O.rmsnorm_fwd(x, w["ln1_scale"], cfg.rms_eps)
    n1 = rb(n1_full)
    n1_qk = n1_full if split_n1 else n1
    q_full, k_full = _heads(n1_qk @ w["wq"], nh, dk), _heads(n1_qk @ w["wk"], nh, dk)
    q_lp, k_lp = rb(q_full), rb(k_full)
    q, k = (q_full, k_full) if split_qk else (q_lp, k_lp)
    v = rb(_heads(n1 @ w["wv"], nh, dk))
    bias, bucket = O.relpos_bias(w["rel_table"], S, not cfg.causal, cfg.num_buckets, cfg.max_distance)
    keep_p = _keep(cfg, O.DROP_ATTN_PROBS, (B, nh, S, S))
    keep_o = _keep(cfg, O.DROP_ATTN_OUT, (B, S, cfg.d_model))
    c_h = attention_fwd(cfg, q, k, v, bias, cfg.causal, keep_p)
    c = _merge(c_h)
    h = x + _mul(c @ w["wo"], keep_o)
    return h, dict(x=x, n1=n1, r1=r1, q=q, k=k, q_lp=q_lp, k_lp=k_lp, v=v, bias=bias, bucket=bucket, keep_p=keep_p,
                   keep_o=keep_o, c_h=c_h, c=c)


def self_attn_bwd(cfg, dh, w, sv, g):
    """dx (unrounded) from dh, the float64 gradient of h; adds wq, wk, wv, wo, rel_table, ln1_scale to g."""
    nh, dk = cfg.n_heads, cfg.d_kv
    dao = rb(dh)
    if sv["keep_o"] is not None:
        dao = rb(dao * sv["keep_o"])
    g["wo"] = _flat(sv["c"]).T @ _flat(dao)
    do = rb(_heads(dao @ w["wo"].T, nh, dk))
    dq, dk_, dv, ds = attention_bwd(cfg, sv["q"], sv["k"], sv["v"], sv["bias"], cfg.causal, sv["keep_p"], sv["c_h"],
                                    do, sv["q_lp"], sv["k_lp"])
    dtable = np.zeros_like(w["rel_table"])
    ds_hij = ds.sum(0)
    for hh in range(nh):
        np.add.at(dtable[:, hh], sv["bucket"].reshape(-1), ds_hij[hh].reshape(-1))
    g["rel_table"] = dtable
    dqf, dkf, dvf = _merge(dq), _merge(dk_), _merge(dv)
    n1 = sv["n1"]
    g["wq"] = _flat(n1).T @ _flat(dqf)
    g["wk"] = _flat(n1).T @ _flat(dkf)
    g["wv"] = _flat(n1).T @ _flat(dvf)
    dn1 = dqf @ w["wq"].T + dkf @ w["wk"].T + dvf @ w["wv"].T
    dx_norm, g["ln1_scale"] = O.rmsnorm_bwd(sv["x"], w["ln1_scale"], sv["r1"], dn1)
    return dh + dx_norm


def cross_attn_fwd(cfg, h1, enc, w):
    """h2 = h1 + CrossAttn(RMSNorm(h1), enc), unrounded."""
    nh, dk, S = cfg.n_heads, cfg.d_kv, cfg.seq
    B, Se = h1.shape[0], enc.shape[1]
    nx, rx = O.rmsnorm_fwd(h1, w["lnx_scale"], cfg.rms_eps)
    nx = rb(nx)
    q = rb(_heads(nx @ w["xq"], nh, dk))
    k = rb(_heads(enc @ w["xk"], nh, dk))
    v = rb(_heads(enc @ w["xv"], nh, dk))
    keep_p = _keep(cfg, O.DROP_CROSS_PROBS, (B, nh, S, Se))
    keep_o = _keep(cfg, O.DROP_CROSS_OUT, (B, S, cfg.d_model))
    c_h = attention_fwd(cfg, q, k, v, None, False, keep_p)
    c = _merge(c_h)
    h2 = h1 + _mul(c @ w["xo"], keep_o)
    return h2, dict(h1=h1, enc=enc, nx=nx, rx=rx, q=q, k=k, v=v, keep_p=keep_p, keep_o=keep_o, c_h=c_h, c=c)


def cross_attn_bwd(cfg, dh2, w, sv, g, round_denc=True):
    """(dh1 unrounded, denc) from dh2; adds xq, xk, xv, xo, lnx_scale to g.  denc is rounded to bf16 as the
    decoder layer's entry point stores it; a stack sums the layers' contributions in float32 (round_denc=False)."""
    nh, dk = cfg.n_heads, cfg.d_kv
    dao = rb(dh2)
    if sv["keep_o"] is not None:
        dao = rb(dao * sv["keep_o"])
    g["xo"] = _flat(sv["c"]).T @ _flat(dao)
    do = rb(_heads(dao @ w["xo"].T, nh, dk))
    dq, dk_, dv, _ = attention_bwd(cfg, sv["q"], sv["k"], sv["v"], None, False, sv["keep_p"], sv["c_h"], do)
    dqf, dkf, dvf = _merge(dq), _merge(dk_), _merge(dv)
    g["xq"] = _flat(sv["nx"]).T @ _flat(dqf)
    g["xk"] = _flat(sv["enc"]).T @ _flat(dkf)
    g["xv"] = _flat(sv["enc"]).T @ _flat(dvf)
    denc = dkf @ w["xk"].T + dvf @ w["xv"].T
    if round_denc:
        denc = rb(denc)
    dh1_norm, g["lnx_scale"] = O.rmsnorm_bwd(sv["h1"], w["lnx_scale"], sv["rx"], dqf @ w["xq"].T)
    return dh2 + dh1_norm, denc


def mlp_fwd(cfg, h, w, round_uw=False):
    """y = h + MLP(RMSNorm(h)), rounded (the block's output is stored in bf16).
    round_uw: the two input projections are stored in bf16 before the activation is applied (what the
    general-shape kernels do; the matrix-unit path applies it to the float32 accumulators)."""
    B, S = h.shape[0], h.shape[1]
    n2, r2 = O.rmsnorm_fwd(h, w["ln2_scale"], cfg.rms_eps)
    n2 = rb(n2)
    keep_h = _keep(cfg, O.DROP_MLP_HIDDEN, (B, S, cfg.d_ff))
    keep_o = _keep(cfg, O.DROP_MLP_OUT, (B, S, cfg.d_model))
    u = n2 @ w["wi0"]
    if round_uw:
        u = rb(u)
    sv = dict(h=h, n2=n2, r2=r2, keep_h=keep_h, keep_o=keep_o)
    if cfg.mlp == "relu":
        sv["a"] = rb(_mul(np.maximum(u, 0.0), keep_h))
    else:
        wl = n2 @ w["wi1"]
        if round_uw:
            wl = rb(wl)
        gl, dgl = _act(cfg, u)
        sv["gp"] = rb(_mul(wl * dgl, keep_h))
        sv["gl"] = rb(_mul(gl, keep_h))
        sv["a"] = rb(_mul(gl * wl, keep_h))
    return rb(h + _mul(sv["a"] @ w["wo_ff"], keep_o)), sv


def mlp_bwd(cfg, dy, w, sv, g):
    """dh (unrounded) from dy (bf16); adds wo_ff, wi0[, wi1], ln2_scale to g."""
    n2 = sv["n2"]
    dyo = dy if sv["keep_o"] is None else rb(dy * sv["keep_o"])
    g["wo_ff"] = _flat(sv["a"]).T @ _flat(dyo)
    da = dyo @ w["wo_ff"].T
    if cfg.mlp == "relu":
        scale = 1.0 / (1.0 - cfg.dropout_rate) if sv["keep_h"] is not None else 1.0
        du = rb(np.where(sv["a"] > 0.0, da * scale, 0.0))
        g["wi0"] = _flat(n2).T @ _flat(du)
        dn2 = du @ w["wi0"].T
    else:
        du, dwl = rb(da * sv["gp"]), rb(da * sv["gl"])
        g["wi0"] = _flat(n2).T @ _flat(du)
        g["wi1"] = _flat(n2).T @ _flat(dwl)
        dn2 = du @ w["wi0"].T + dwl @ w["wi1"].T
    dh_norm, g["ln2_scale"] = O.rmsnorm_bwd(sv["h"], w["ln2_scale"], sv["r2"], dn2)
    return dy + dh_norm


# ------------------------------------------------------------------------------ whole layers
def block_model(cfg, x, w, dy, split_qk=False, split_n1=False, round_uw=False):
    """(y, dx, grads) of one block under ideal bf16-operand arithmetic.  x, dy and w hold
    bf16-representable values."""
    h, sa = self_attn_fwd(cfg, x, w, split_qk, split_n1)
    y, sm = mlp_fwd(cfg, h, w, round_uw)
    g = {}
    dh = mlp_bwd(cfg, dy, w, sm, g)
    dx = rb(self_attn_bwd(cfg, dh, w, sa, g))
    return y, dx, g


def decoder_block_model(cfg, x, enc, w, dy, round_uw=False):
    """(y, dx, denc, grads) of one decoder layer under ideal bf16-operand arithmetic."""
    h1, sa = self_attn_fwd(cfg, x, w)
    h2, sx = cross_attn_fwd(cfg, h1, enc, w)
    y, sm = mlp_fwd(cfg, h2, w, round_uw)
    g = {}
    dh2 = mlp_bwd(cfg, dy, w, sm, g)
    dh1, denc = cross_attn_bwd(cfg, dh2, w, sx, g)
    dx = rb(self_attn_bwd(cfg, dh1, w, sa, g))
    return y, dx, denc, g


# ------------------------------------------------------------------------------ stacks
def _layer_fwd(cfg, x, w, enc, round_uw):
    h, sa = self_attn_fwd(cfg, x, w)
    sx = None
    if enc is not None:
        h, sx = cross_attn_fwd(cfg, h, enc, w)
    y, sm = mlp_fwd(cfg, h, w, round_uw)
    return y, (sa, sx, sm)


def _layer_bwd(cfg, dy, w, saved):
    """(dx rounded to bf16 -- the residual stream crosses layer boundaries in the storage type --,
    denc unrounded or None, gradients)."""
    sa, sx, sm = saved
    g = {}
    dh = mlp_bwd(cfg, dy, w, sm, g)
    denc = None
    if sx is not None:
        dh, denc = cross_attn_bwd(cfg, dh, w, sx, g, round_denc=False)
    return rb(self_attn_bwd(cfg, dh, w, sa, g)), denc, g


def _head(cfg, x_last, final_scale, emb_or_w, tied, targets, z_loss, site):
    """Final norm, logits, loss and the gradients of the head.  Returns (loss, dx_last rounded, dfinal_scale,
    dW of the output matrix (or of the tied embedding), nf)."""
    s = cfg.d_model ** -0.5 if tied else 1.0
    gf = rb(final_scale * s) if tied else final_scale          # tied: the factor rides on the (stored) scale
    nf, rf = O.rmsnorm_fwd(x_last, gf, cfg.rms_eps)
    m_final = O._token_scale(cfg, site, nf.shape)
    nf = rb(rb(nf) * m_final) if not np.isscalar(m_final) else rb(nf)
    wmat = emb_or_w.T if tied else emb_or_w                    # [d, V]
    logits = rb(nf @ wmat)
    loss, lse, n = O.xent_zloss(logits, targets, z_loss)
    dlogits = rb(O.xent_zloss_grad(logits, targets, lse, z_loss, n))
    dw = _flat(nf).T @ _flat(dlogits)                          # [d, V]
    dnf = dlogits @ wmat.T
    dx, dgf = O.rmsnorm_bwd(x_last, gf, rf, dnf * m_final)
    return loss, rb(dx), dgf * s, (dw.T if tied else dw)


def stack_model(sc, tokens, targets, w, round_uw=False):
    """(loss, gradients nested like the oracle's stack_loss_grad) under ideal bf16-operand arithmetic."""
    cfg = sc.block
    x = w["embedding"][tokens]
    m_embed = O._token_scale(cfg, O.DROP_EMBED, x.shape)
    if not np.isscalar(m_embed):
        x = rb(x * m_embed)
    saved = []
    for l, lw in enumerate(w["layers"]):
        wl = dict(lw, rel_table=w["rel_table"])
        x, sv = _layer_fwd(O._with_layer_seed(cfg, l), x, wl, None, round_uw)
        saved.append(sv)
    loss, dx, dgf, dw = _head(cfg, x, w["final_scale"], w["embedding"] if sc.tied_logits else w["logits_w"],
                              sc.tied_logits, targets, sc.z_loss, O.DROP_FINAL)
    g = {"layers": [None] * sc.n_layers, "embedding": np.zeros_like(w["embedding"]), "final_scale": dgf,
         "rel_table": np.zeros_like(w["rel_table"])}
    if sc.tied_logits:
        g["embedding"] += dw
    else:
        g["logits_w"] = dw
    for l in range(sc.n_layers - 1, -1, -1):
        wl = dict(w["layers"][l], rel_table=w["rel_table"])
        dx, _, gl = _layer_bwd(O._with_layer_seed(cfg, l), dx, wl, saved[l])
        g["rel_table"] += gl.pop("rel_table")
        g["layers"][l] = gl
    if not np.isscalar(m_embed):
        dx = rb(dx * m_embed)
    np.add.at(g["embedding"], tokens.reshape(-1), _flat(dx))
    return loss, g


def encdec_model(ec, enc_tokens, dec_tokens, targets, w, round_uw=False):
    """(loss, gradients nested like the oracle's encdec_loss_grad) under ideal bf16-operand arithmetic."""
    e, d = ec.enc_block, ec.dec_block
    x = w["embedding"][enc_tokens]
    me_embed = O._token_scale(e, O.DROP_EMBED, x.shape)
    if not np.isscalar(me_embed):
        x = rb(x * me_embed)
    enc_saved = []
    for l, lw in enumerate(w["enc_layers"]):
        x, sv = _layer_fwd(O._with_layer_seed(e, l), x, dict(lw, rel_table=w["enc_rel_table"]), None, round_uw)
        enc_saved.append(sv)
    xe_last = x
    enc_out, enc_rf = O.rmsnorm_fwd(x, w["enc_final_scale"], e.rms_eps)
    me_final = O._token_scale(e, O.DROP_FINAL, enc_out.shape)
    enc_out = rb(rb(enc_out) * me_final) if not np.isscalar(me_final) else rb(enc_out)
    x = w["embedding"][dec_tokens]
    md_embed = O._token_scale(d, O.DROP_DEC_EMBED, x.shape)
    if not np.isscalar(md_embed):
        x = rb(x * md_embed)
    dec_saved = []
    for l, lw in enumerate(w["dec_layers"]):
        x, sv = _layer_fwd(O._with_layer_seed(d, ec.n_enc_layers + l), x, dict(lw, rel_table=w["dec_rel_table"]),
                           enc_out, round_uw)
        dec_saved.append(sv)
    loss, dx, dgf, dw = _head(d, x, w["dec_final_scale"], w["embedding"] if ec.tied_logits else w["logits_w"],
                              ec.tied_logits, targets, ec.z_loss, O.DROP_DEC_FINAL)
    g = {"embedding": np.zeros_like(w["embedding"]), "enc_layers": [None] * ec.n_enc_layers,
         "dec_layers": [None] * ec.n_dec_layers, "dec_final_scale": dgf,
         "dec_rel_table": np.zeros_like(w["dec_rel_table"]), "enc_rel_table": np.zeros_like(w["enc_rel_table"])}
    if ec.tied_logits:
        g["embedding"] += dw
    else:
        g["logits_w"] = dw
    denc_out = 0.0
    for l in range(ec.n_dec_layers - 1, -1, -1):
        wl = dict(w["dec_layers"][l], rel_table=w["dec_rel_table"])
        dx, denc_l, gl = _layer_bwd(O._with_layer_seed(d, ec.n_enc_layers + l), dx, wl, dec_saved[l])
        denc_out = denc_out + denc_l
        g["dec_rel_table"] += gl.pop("rel_table")
        g["dec_layers"][l] = gl
    if not np.isscalar(md_embed):
        dx = rb(dx * md_embed)
    np.add.at(g["embedding"], dec_tokens.reshape(-1), _flat(dx))
    dx, g["enc_final_scale"] = O.rmsnorm_bwd(xe_last, w["enc_final_scale"], enc_rf, denc_out * me_final)
    dx = rb(dx)
    for l in range(ec.n_enc_layers - 1, -1, -1):
        wl = dict(w["enc_layers"][l], rel_table=w["enc_rel_table"])
        dx, _, gl = _layer_bwd(O._with_layer_seed(e, l), dx, wl, enc_saved[l])
        g["enc_rel_table"] += gl.pop("rel_table")
        g["enc_layers"][l] = gl
    if not np.isscalar(me_embed):
        dx = rb(dx * me_embed)
    np.add.at(g["embedding"], enc_tokens.reshape(-1), _flat(dx))
    return loss, g


def rel_err(a: np.ndarray, ref: np.ndarray):
    """(max, mean) of |a - ref| / max(|ref|, RMS(ref)): the metric of the parity tests."""
    rms = float(np.sqrt(np.mean(ref * ref)))
    if rms == 0.0:
        return float(np.abs(a).max()), float(np.abs(a).mean())
    e = np.abs(a - ref) / np.maximum(np.abs(ref), rms)
    return float(e.max()), float(e.mean())


def block_floor(cfg, x, w, dy, ref=None, **kw):
    """Per-tensor (max, mean) error of block_model against the float64 oracle: {"y", "dx", weight names}.
    ref: (y, dx, grads) of the oracle when the caller already has them."""
    if ref is None:
        y, saved = O.block_fwd(cfg, x, w)
        dx, g = O.block_bwd(cfg, dy, w, saved)
    else:
        y, dx, g = ref
    my, mdx, mg = block_model(cfg, x, w, dy, **kw)
    out = {"y": rel_err(my, y), "dx": rel_err(mdx, dx)}
    out.update({k: rel_err(mg[k], g[k]) for k in g})
    return out


def decoder_block_floor(cfg, x, enc, w, dy, ref=None, **kw):
    """The same for a decoder layer: {"y", "dx", "denc", weight names}.  ref: (y, dx, denc, grads)."""
    if ref is None:
        y, saved = O.decoder_block_fwd(cfg, x, enc, w)
        dx, denc, g = O.decoder_block_bwd(cfg, dy, w, saved)
    else:
        y, dx, denc, g = ref
    my, mdx, mde, mg = decoder_block_model(cfg, x, enc, w, dy, **kw)
    out = {"y": rel_err(my, y), "dx": rel_err(mdx, dx), "denc": rel_err(mde, denc)}
    out.update({k: rel_err(mg[k], g[k]) for k in g})
    return out
