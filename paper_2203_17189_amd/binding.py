"""ctypes binding of libt5mi.so.  Argument marshalling only; torch supplies device memory and
streams.  There is no CPU fallback: a missing library raises."""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

WEIGHT_NAMES = ("ln1_scale", "wq", "wk", "wv", "wo", "rel_table", "ln2_scale", "wi0", "wi1", "wo_ff")
CROSS_WEIGHT_NAMES = ("lnx_scale", "xq", "xk", "xv", "xo")
T5_F32, T5_BF16 = 0, 1
MLP_KINDS = {"geglu_tanh": 0, "relu": 1, "geglu_erf": 2}


class T5Error(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: status {status} ({t5_status_string(status)})")
        self.status = status


class _Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("batch", "seq", "d_model", "n_heads", "d_kv", "d_ff", "num_buckets",
                                         "max_distance", "causal", "dtype")] + \
               [("rms_eps", C.c_float), ("attn_scale", C.c_float), ("mlp_kind", C.c_int32),
                ("dropout_rate", C.c_float), ("dropout_seed_lo", C.c_uint32), ("dropout_seed_hi", C.c_uint32),
                ("deterministic", C.c_int32)]


class _Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_NAMES]


class _Grads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_NAMES]


class _CrossWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in CROSS_WEIGHT_NAMES]


class _CrossGrads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in CROSS_WEIGHT_NAMES]


class _StackCfg(C.Structure):
    _fields_ = [("block", _Cfg), ("n_layers", C.c_int32), ("vocab", C.c_int32), ("tied_logits", C.c_int32),
                ("remat", C.c_int32), ("z_loss", C.c_float)]


class _StackWeights(C.Structure):
    _fields_ = [("embedding", C.c_void_p), ("rel_table", C.c_void_p), ("layers", C.POINTER(_Weights)),
                ("final_scale", C.c_void_p), ("logits_w", C.c_void_p)]


class _StackGrads(C.Structure):
    _fields_ = [("embedding", C.c_void_p), ("rel_table", C.c_void_p), ("layers", C.POINTER(_Grads)),
                ("final_scale", C.c_void_p), ("logits_w", C.c_void_p)]


class _EncDecCfg(C.Structure):
    _fields_ = [("enc_block", _Cfg), ("dec_block", _Cfg), ("n_enc_layers", C.c_int32), ("n_dec_layers", C.c_int32),
                ("vocab", C.c_int32), ("tied_logits", C.c_int32), ("remat", C.c_int32), ("z_loss", C.c_float)]


class _EncDecWeights(C.Structure):
    _fields_ = [("embedding", C.c_void_p), ("enc_rel_table", C.c_void_p), ("enc_layers", C.POINTER(_Weights)),
                ("enc_final_scale", C.c_void_p), ("dec_rel_table", C.c_void_p), ("dec_layers", C.POINTER(_Weights)),
                ("dec_cross", C.POINTER(_CrossWeights)), ("dec_final_scale", C.c_void_p), ("logits_w", C.c_void_p)]


class _EncDecGrads(C.Structure):
    _fields_ = [("embedding", C.c_void_p), ("enc_rel_table", C.c_void_p), ("enc_layers", C.POINTER(_Grads)),
                ("enc_final_scale", C.c_void_p), ("dec_rel_table", C.c_void_p), ("dec_layers", C.POINTER(_Grads)),
                ("dec_cross", C.POINTER(_CrossGrads)), ("dec_final_scale", C.c_void_p), ("logits_w", C.c_void_p)]


class _AfTensor(C.Structure):
    _fields_ = [("param", C.c_void_p), ("grad", C.c_void_p), ("v_row", C.c_void_p), ("v_col", C.c_void_p),
                ("v_full", C.c_void_p), ("rows", C.c_int64), ("cols", C.c_int64), ("factored", C.c_int32),
                ("bf16_copy_out", C.c_void_p), ("m", C.c_void_p)]


class _AfCfg(C.Structure):
    _fields_ = [("lr", C.c_float), ("decay_pow", C.c_float), ("eps1", C.c_float), ("eps2", C.c_float),
                ("clip", C.c_float), ("scale_by_param", C.c_int32), ("step", C.c_int32), ("beta1", C.c_float),
                ("weight_decay", C.c_float)]


def lib_path() -> str:
    return os.path.join(_HERE, "libt5mi.so")


def lib() -> C.CDLL:
    """Load libt5mi.so (building it first if it is not there).  Raises if that fails."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        from . import build as _build
        _build.build(verbose=False)
    L = C.CDLL(path)
    vp, i32, i64, sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
    L.t5_status_string.restype = C.c_char_p
    L.t5_status_string.argtypes = [i32]
    L.t5_relpos_bucket.restype = i32
    L.t5_relpos_bucket.argtypes = [vp, vp, i64, i32, i32, i32, vp]
    L.t5_dropout_keep.restype = i32
    L.t5_dropout_keep.argtypes = [C.c_uint64, i32, C.c_float, i64, i64, vp, vp]
    L.t5_block_kernel_path.restype = i32
    L.t5_block_kernel_path.argtypes = [C.POINTER(_Cfg), i32]
    L.t5_block_stash_bytes.restype = sz
    L.t5_block_stash_bytes.argtypes = [C.POINTER(_Cfg)]
    L.t5_block_workspace_bytes.restype = sz
    L.t5_block_workspace_bytes.argtypes = [C.POINTER(_Cfg)]
    L.t5_block_fwd.restype = i32
    L.t5_block_fwd.argtypes = [C.POINTER(_Cfg), vp, C.POINTER(_Weights), vp, vp, vp, sz, vp]
    L.t5_block_bwd.restype = i32
    L.t5_block_bwd.argtypes = [C.POINTER(_Cfg), vp, vp, C.POINTER(_Weights), vp, vp, C.POINTER(_Grads), i32,
                               vp, sz, vp]
    L.t5_decoder_block_stash_bytes.restype = sz
    L.t5_decoder_block_stash_bytes.argtypes = [C.POINTER(_Cfg), C.c_int32]
    L.t5_decoder_block_workspace_bytes.restype = sz
    L.t5_decoder_block_workspace_bytes.argtypes = [C.POINTER(_Cfg), C.c_int32]
    L.t5_decoder_block_fwd.restype = i32
    L.t5_decoder_block_fwd.argtypes = [C.POINTER(_Cfg), C.c_int32, vp, vp, C.POINTER(_Weights),
                                       C.POINTER(_CrossWeights), vp, vp, vp, sz, vp]
    L.t5_decoder_block_bwd.restype = i32
    L.t5_decoder_block_bwd.argtypes = [C.POINTER(_Cfg), C.c_int32, vp, vp, vp, C.POINTER(_Weights),
                                       C.POINTER(_CrossWeights), vp, vp, vp, C.POINTER(_Grads),
                                       C.POINTER(_CrossGrads), i32, vp, sz, vp]
    L.t5_stack_workspace_bytes.restype = sz
    L.t5_stack_workspace_bytes.argtypes = [C.POINTER(_StackCfg)]
    L.t5_stack_loss_and_grad.restype = i32
    L.t5_stack_loss_and_grad.argtypes = [C.POINTER(_StackCfg), vp, vp, C.POINTER(_StackWeights), vp,
                                         C.POINTER(_StackGrads), i32, vp, sz, vp]
    L.t5_encdec_workspace_bytes.restype = sz
    L.t5_encdec_workspace_bytes.argtypes = [C.POINTER(_EncDecCfg)]
    L.t5_encdec_loss_and_grad.restype = i32
    L.t5_encdec_loss_and_grad.argtypes = [C.POINTER(_EncDecCfg), vp, vp, vp, C.POINTER(_EncDecWeights), vp,
                                          C.POINTER(_EncDecGrads), i32, vp, sz, vp]
    L.adafactor_workspace_bytes.restype = sz
    L.adafactor_workspace_bytes.argtypes = [i64, i64, i32]
    L.adafactor_step.restype = i32
    L.adafactor_step.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, C.POINTER(_AfCfg), vp, vp, sz, vp]
    L.adafactor_step_static.restype = i32
    L.adafactor_step_static.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, C.POINTER(_AfCfg), vp, vp]
    L.adafactor_multi_workspace_bytes.restype = sz
    L.adafactor_multi_workspace_bytes.argtypes = [C.POINTER(_AfTensor), i32]
    L.adafactor_step_multi.restype = i32
    L.adafactor_step_multi.argtypes = [C.POINTER(_AfTensor), i32, C.POINTER(_AfCfg), vp, sz, vp]
    L.t5_gemm_bf16.restype = i32
    L.t5_gemm_bf16.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp]
    L.t5_wgrad_overlap_enable.restype = i32
    L.t5_wgrad_overlap_enable.argtypes = [i32]
    L.t5_step_timing_enable.restype = None
    L.t5_step_timing_enable.argtypes = [i32]
    L.t5_mfma_peak_probe.restype = i32
    L.t5_mfma_peak_probe.argtypes = [i32, i32, i32, vp, vp]
    L.t5_step_timing_read.restype = i32
    L.t5_step_timing_read.argtypes = [C.POINTER(C.c_char_p), C.POINTER(C.c_float), C.POINTER(i32), i32]
    _LIB = L
    return L


def t5_status_string(status: int) -> str:
    return lib().t5_status_string(int(status)).decode()


def _cfg_struct(cfg) -> _Cfg:
    dt = cfg.dtype
    if isinstance(dt, str):
        dt = {"f32": T5_F32, "bf16": T5_BF16}[dt]
    return _Cfg(cfg.batch, cfg.seq, cfg.d_model, cfg.n_heads, cfg.d_kv, cfg.d_ff, cfg.num_buckets,
                cfg.max_distance, int(bool(cfg.causal)), int(dt), float(cfg.rms_eps), float(cfg.attn_scale),
                MLP_KINDS[getattr(cfg, "mlp", "geglu_tanh")], float(getattr(cfg, "dropout_rate", 0.0)),
                int(getattr(cfg, "dropout_seed", 0)) & 0xFFFFFFFF, (int(getattr(cfg, "dropout_seed", 0)) >> 32) & 0xFFFFFFFF,
                int(bool(getattr(cfg, "deterministic", False))))


def _torch_dtype(cfg):
    dt = cfg.dtype
    return torch.bfloat16 if dt in ("bf16", T5_BF16) else torch.float32


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check_tensor(t, dtype, numel, name):
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype or t.numel() != numel:
        raise ValueError(f"{name}: need a contiguous cuda tensor of {dtype} with {numel} elements, "
                         f"got {t.dtype} {tuple(t.shape)} on {t.device}")


def t5_relpos_bucket(rel_pos: torch.Tensor, bidirectional: bool, num_buckets: int = 32,
                     max_distance: int = 128, out: torch.Tensor | None = None) -> torch.Tensor:
    _check_tensor(rel_pos, torch.int32, rel_pos.numel(), "rel_pos")
    if out is None:
        out = torch.empty_like(rel_pos)
    rc = lib().t5_relpos_bucket(_ptr(rel_pos), _ptr(out), rel_pos.numel(), int(bool(bidirectional)),
                                int(num_buckets), int(max_distance), _stream())
    if rc:
        raise T5Error(rc, "t5_relpos_bucket")
    return out


def t5_dropout_keep(seed: int, site: int, rate: float, rows: int, cols: int) -> torch.Tensor:
    """uint8 [rows, cols] keep mask (1 = kept) of a dropout site, as the block's kernels regenerate it."""
    out = torch.empty(rows, cols, dtype=torch.uint8, device="cuda")
    rc = lib().t5_dropout_keep(C.c_uint64(int(seed) & (2 ** 64 - 1)), int(site), float(rate), int(rows), int(cols),
                               _ptr(out), _stream())
    if rc:
        raise T5Error(rc, "t5_dropout_keep")
    return out


PATH_MFMA_GEMM, PATH_MFMA_ATTN_FWD, PATH_MFMA_ATTN_BWD, PATH_MFMA_CROSS_ATTN = 1, 2, 4, 8


def t5_block_kernel_path(cfg) -> int:
    """Bit mask of the kernel families the configuration runs on (host-side query; -1: invalid configuration)."""
    return int(lib().t5_block_kernel_path(C.byref(_cfg_struct(cfg)), int(getattr(cfg, "enc_seq", 0))))


def t5_block_stash_bytes(cfg) -> int:
    return int(lib().t5_block_stash_bytes(C.byref(_cfg_struct(cfg))))


def t5_block_workspace_bytes(cfg) -> int:
    return int(lib().t5_block_workspace_bytes(C.byref(_cfg_struct(cfg))))


def _block_names(cfg, names=WEIGHT_NAMES):
    """Tensor names of a block: the ungated ReLU feed-forward has no wi1."""
    return tuple(n for n in names if not (n == "wi1" and getattr(cfg, "mlp", "geglu_tanh") == "relu"))


def _addr(d, n):
    t = d.get(n)
    return None if t is None else t.data_ptr()


def _weights_struct(cfg, weights) -> _Weights:
    dt = _torch_dtype(cfg)
    inner = cfg.n_heads * cfg.d_kv
    shapes = {"ln1_scale": cfg.d_model, "ln2_scale": cfg.d_model, "wq": cfg.d_model * inner,
              "wk": cfg.d_model * inner, "wv": cfg.d_model * inner, "wo": inner * cfg.d_model,
              "rel_table": cfg.num_buckets * cfg.n_heads, "wi0": cfg.d_model * cfg.d_ff,
              "wi1": cfg.d_model * cfg.d_ff, "wo_ff": cfg.d_ff * cfg.d_model}
    names = _block_names(cfg)
    for n in names:
        _check_tensor(weights[n], dt, shapes[n], n)
    return _Weights(*[(_addr(weights, n) if n in names else None) for n in WEIGHT_NAMES])


def _byte_buffer(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def t5_block_fwd(cfg, x, weights, y=None, stash=None, workspace=None):
    """Returns (y, stash).  stash/workspace are uint8 cuda tensors (allocated here if None)."""
    cs = _cfg_struct(cfg)
    dt = _torch_dtype(cfg)
    n = cfg.batch * cfg.seq * cfg.d_model
    _check_tensor(x, dt, n, "x")
    ws = _weights_struct(cfg, weights)
    if y is None:
        y = torch.empty_like(x)
    _check_tensor(y, dt, n, "y")
    if stash is None:
        stash = _byte_buffer(lib().t5_block_stash_bytes(C.byref(cs)), x.device)
    if workspace is None:
        workspace = _byte_buffer(lib().t5_block_workspace_bytes(C.byref(cs)), x.device)
    rc = lib().t5_block_fwd(C.byref(cs), _ptr(x), C.byref(ws), _ptr(y), _ptr(stash), _ptr(workspace),
                            workspace.numel(), _stream())
    if rc:
        raise T5Error(rc, "t5_block_fwd")
    return y, stash


def alloc_grads(cfg, weights) -> dict:
    return {n: torch.zeros(weights[n].shape, dtype=torch.float32, device=weights[n].device)
            for n in _block_names(cfg)}


def t5_block_bwd(cfg, dy, x, weights, stash, dx=None, grads=None, accumulate=False, workspace=None):
    """Returns (dx, grads); grads is a dict of float32 tensors shaped like the weights."""
    cs = _cfg_struct(cfg)
    dt = _torch_dtype(cfg)
    n = cfg.batch * cfg.seq * cfg.d_model
    _check_tensor(dy, dt, n, "dy")
    _check_tensor(x, dt, n, "x")
    ws = _weights_struct(cfg, weights)
    if dx is None:
        dx = torch.empty_like(dy)
    _check_tensor(dx, dt, n, "dx")
    if grads is None:
        grads = alloc_grads(cfg, weights)
    for nme in _block_names(cfg):
        _check_tensor(grads[nme], torch.float32, weights[nme].numel(), "grad " + nme)
    gs = _Grads(*[_addr(grads, nme) for nme in WEIGHT_NAMES])
    if workspace is None:
        workspace = _byte_buffer(lib().t5_block_workspace_bytes(C.byref(cs)), x.device)
    rc = lib().t5_block_bwd(C.byref(cs), _ptr(dy), _ptr(x), C.byref(ws), _ptr(stash), _ptr(dx), C.byref(gs),
                            int(bool(accumulate)), _ptr(workspace), workspace.numel(), _stream())
    if rc:
        raise T5Error(rc, "t5_block_bwd")
    return dx, grads


def t5_decoder_block_stash_bytes(cfg) -> int:
    return int(lib().t5_decoder_block_stash_bytes(C.byref(_cfg_struct(cfg)), int(cfg.enc_seq)))


def t5_decoder_block_workspace_bytes(cfg) -> int:
    return int(lib().t5_decoder_block_workspace_bytes(C.byref(_cfg_struct(cfg)), int(cfg.enc_seq)))


def _cross_weights_struct(cfg, weights) -> _CrossWeights:
    dt = _torch_dtype(cfg)
    inner = cfg.n_heads * cfg.d_kv
    shapes = {"lnx_scale": cfg.d_model, "xq": cfg.d_model * inner, "xk": cfg.d_model * inner,
              "xv": cfg.d_model * inner, "xo": inner * cfg.d_model}
    for n in CROSS_WEIGHT_NAMES:
        _check_tensor(weights[n], dt, shapes[n], n)
    return _CrossWeights(*[weights[n].data_ptr() for n in CROSS_WEIGHT_NAMES])


def t5_decoder_block_fwd(cfg, x, enc, weights, y=None, stash=None, workspace=None):
    """Decoder layer with cross-attention over enc [batch, cfg.enc_seq, d_model].  weights holds the
    block's ten tensors and the five cross-attention tensors.  Returns (y, stash)."""
    cs = _cfg_struct(cfg)
    dt = _torch_dtype(cfg)
    n = cfg.batch * cfg.seq * cfg.d_model
    _check_tensor(x, dt, n, "x")
    _check_tensor(enc, dt, cfg.batch * cfg.enc_seq * cfg.d_model, "enc")
    ws = _weights_struct(cfg, weights)
    xs = _cross_weights_struct(cfg, weights)
    if y is None:
        y = torch.empty_like(x)
    _check_tensor(y, dt, n, "y")
    es = int(cfg.enc_seq)
    if stash is None:
        stash = _byte_buffer(lib().t5_decoder_block_stash_bytes(C.byref(cs), es), x.device)
    if workspace is None:
        workspace = _byte_buffer(lib().t5_decoder_block_workspace_bytes(C.byref(cs), es), x.device)
    rc = lib().t5_decoder_block_fwd(C.byref(cs), es, _ptr(x), _ptr(enc), C.byref(ws), C.byref(xs), _ptr(y),
                                    _ptr(stash), _ptr(workspace), workspace.numel(), _stream())
    if rc:
        raise T5Error(rc, "t5_decoder_block_fwd")
    return y, stash


def alloc_decoder_grads(cfg, weights) -> dict:
    return {n: torch.zeros(weights[n].shape, dtype=torch.float32, device=weights[n].device)
            for n in _block_names(cfg) + CROSS_WEIGHT_NAMES}


def t5_decoder_block_bwd(cfg, dy, x, enc, weights, stash, dx=None, denc=None, grads=None, accumulate=False,
                         workspace=None):
    """Returns (dx, denc, grads); grads is a dict of float32 tensors shaped like the fifteen weights."""
    cs = _cfg_struct(cfg)
    dt = _torch_dtype(cfg)
    n = cfg.batch * cfg.seq * cfg.d_model
    ne = cfg.batch * cfg.enc_seq * cfg.d_model
    _check_tensor(dy, dt, n, "dy")
    _check_tensor(x, dt, n, "x")
    _check_tensor(enc, dt, ne, "enc")
    ws = _weights_struct(cfg, weights)
    xs = _cross_weights_struct(cfg, weights)
    if dx is None:
        dx = torch.empty_like(dy)
    if denc is None:
        denc = torch.empty_like(enc)
    _check_tensor(dx, dt, n, "dx")
    _check_tensor(denc, dt, ne, "denc")
    if grads is None:
        grads = alloc_decoder_grads(cfg, weights)
    for nme in _block_names(cfg) + CROSS_WEIGHT_NAMES:
        _check_tensor(grads[nme], torch.float32, weights[nme].numel(), "grad " + nme)
    gs = _Grads(*[_addr(grads, nme) for nme in WEIGHT_NAMES])
    gx = _CrossGrads(*[grads[nme].data_ptr() for nme in CROSS_WEIGHT_NAMES])
    es = int(cfg.enc_seq)
    if workspace is None:
        workspace = _byte_buffer(lib().t5_decoder_block_workspace_bytes(C.byref(cs), es), x.device)
    rc = lib().t5_decoder_block_bwd(C.byref(cs), es, _ptr(dy), _ptr(x), _ptr(enc), C.byref(ws), C.byref(xs),
                                    _ptr(stash), _ptr(dx), _ptr(denc), C.byref(gs), C.byref(gx),
                                    int(bool(accumulate)), _ptr(workspace), workspace.numel(), _stream())
    if rc:
        raise T5Error(rc, "t5_decoder_block_bwd")
    return dx, denc, grads


LAYER_WEIGHT_NAMES = tuple(n for n in WEIGHT_NAMES if n != "rel_table")


def _stack_cfg_struct(sc) -> _StackCfg:
    return _StackCfg(_cfg_struct(sc.block), int(sc.n_layers), int(sc.vocab), int(bool(sc.tied_logits)),
                     int(bool(sc.remat)), float(sc.z_loss))


def t5_stack_workspace_bytes(sc) -> int:
    return int(lib().t5_stack_workspace_bytes(C.byref(_stack_cfg_struct(sc))))


def alloc_stack_grads(sc, weights) -> dict:
    """float32 zero tensors shaped like the stack's weights: {"embedding", "rel_table", "final_scale",
    "logits_w" (untied), "layers": [dict per layer]}."""
    z = lambda t: torch.zeros(t.shape, dtype=torch.float32, device=t.device)
    g = {k: z(weights[k]) for k in ("embedding", "rel_table", "final_scale")}
    if not sc.tied_logits:
        g["logits_w"] = z(weights["logits_w"])
    g["layers"] = [{n: z(lw[n]) for n in _block_names(sc.block, LAYER_WEIGHT_NAMES)} for lw in weights["layers"]]
    return g


def t5_stack_loss_and_grad(sc, tokens, targets, weights, grads=None, want_grads=True, accumulate=False,
                           workspace=None, loss=None):
    """Loss (and gradients) of a stack of blocks with embedding, final norm, logits and cross-entropy with
    z-loss.  weights: {"embedding", "rel_table", "final_scale", "logits_w" (untied), "layers": [dict of the
    block's tensors without rel_table, per layer]}.  Returns (loss tensor of one float32, grads or None)."""
    b = sc.block
    cs = _stack_cfg_struct(sc)
    dt = _torch_dtype(b)
    n_tok = b.batch * b.seq
    _check_tensor(tokens, torch.int32, n_tok, "tokens")
    _check_tensor(targets, torch.int32, n_tok, "targets")
    _check_tensor(weights["embedding"], dt, sc.vocab * b.d_model, "embedding")
    _check_tensor(weights["rel_table"], dt, b.num_buckets * b.n_heads, "rel_table")
    _check_tensor(weights["final_scale"], dt, b.d_model, "final_scale")
    if not sc.tied_logits:
        _check_tensor(weights["logits_w"], dt, sc.vocab * b.d_model, "logits_w")
    if len(weights["layers"]) != sc.n_layers:
        raise ValueError("weights['layers'] must hold n_layers dicts")
    lw = (_Weights * sc.n_layers)()
    for l, d in enumerate(weights["layers"]):
        lw[l] = _weights_struct(b, dict(d, rel_table=weights["rel_table"]))
    ws = _StackWeights(weights["embedding"].data_ptr(), weights["rel_table"].data_ptr(), lw,
                       weights["final_scale"].data_ptr(),
                       None if sc.tied_logits else weights["logits_w"].data_ptr())
    gs_ref = None
    if want_grads:
        if grads is None:
            grads = alloc_stack_grads(sc, weights)
        names = ["embedding", "rel_table", "final_scale"] + ([] if sc.tied_logits else ["logits_w"])
        for nme in names:
            _check_tensor(grads[nme], torch.float32, weights[nme].numel(), "grad " + nme)
        lg = (_Grads * sc.n_layers)()
        for l, d in enumerate(grads["layers"]):
            for nme in _block_names(b, LAYER_WEIGHT_NAMES):
                _check_tensor(d[nme], torch.float32, weights["layers"][l][nme].numel(), f"grad layer {l} {nme}")
            lg[l] = _Grads(*[(_addr(d, nme) if nme != "rel_table" else grads["rel_table"].data_ptr())
                             for nme in WEIGHT_NAMES])
        gs = _StackGrads(grads["embedding"].data_ptr(), grads["rel_table"].data_ptr(), lg,
                         grads["final_scale"].data_ptr(), None if sc.tied_logits else grads["logits_w"].data_ptr())
        gs_ref = C.byref(gs)
    else:
        grads = None
    if loss is None:
        loss = torch.zeros(1, dtype=torch.float32, device=tokens.device)
    if workspace is None:
        workspace = _byte_buffer(lib().t5_stack_workspace_bytes(C.byref(cs)), tokens.device)
    rc = lib().t5_stack_loss_and_grad(C.byref(cs), _ptr(tokens), _ptr(targets), C.byref(ws), _ptr(loss), gs_ref,
                                      int(bool(accumulate)), _ptr(workspace), workspace.numel(), _stream())
    if rc:
        raise T5Error(rc, "t5_stack_loss_and_grad")
    return loss, grads


def _encdec_cfg_struct(ec) -> _EncDecCfg:
    return _EncDecCfg(_cfg_struct(ec.enc_block), _cfg_struct(ec.dec_block), int(ec.n_enc_layers),
                      int(ec.n_dec_layers), int(ec.vocab), int(bool(ec.tied_logits)), int(bool(ec.remat)),
                      float(ec.z_loss))


def t5_encdec_workspace_bytes(ec) -> int:
    return int(lib().t5_encdec_workspace_bytes(C.byref(_encdec_cfg_struct(ec))))


_ENCDEC_FLAT = ("embedding", "enc_rel_table", "enc_final_scale", "dec_rel_table", "dec_final_scale")


def alloc_encdec_grads(ec, weights) -> dict:
    z = lambda t: torch.zeros(t.shape, dtype=torch.float32, device=t.device)
    g = {k: z(weights[k]) for k in _ENCDEC_FLAT}
    if not ec.tied_logits:
        g["logits_w"] = z(weights["logits_w"])
    names = _block_names(ec.enc_block, LAYER_WEIGHT_NAMES)
    g["enc_layers"] = [{n: z(lw[n]) for n in names} for lw in weights["enc_layers"]]
    g["dec_layers"] = [{n: z(lw[n]) for n in names + CROSS_WEIGHT_NAMES} for lw in weights["dec_layers"]]
    return g


def t5_encdec_loss_and_grad(ec, enc_tokens, dec_tokens, targets, weights, grads=None, want_grads=True,
                            accumulate=False, workspace=None, loss=None):
    """Loss (and gradients) of the encoder-decoder model.  weights: {"embedding", "enc_rel_table",
    "enc_layers": [block dicts without rel_table], "enc_final_scale", "dec_rel_table", "dec_layers": [block +
    cross-attention dicts without rel_table], "dec_final_scale", "logits_w" (untied)}.
    Returns (loss tensor of one float32, grads or None)."""
    e, d = ec.enc_block, ec.dec_block
    cs = _encdec_cfg_struct(ec)
    dt = _torch_dtype(d)
    _check_tensor(enc_tokens, torch.int32, e.batch * e.seq, "enc_tokens")
    _check_tensor(dec_tokens, torch.int32, d.batch * d.seq, "dec_tokens")
    _check_tensor(targets, torch.int32, d.batch * d.seq, "targets")
    _check_tensor(weights["embedding"], dt, ec.vocab * d.d_model, "embedding")
    for nme, cfgb in (("enc_rel_table", e), ("dec_rel_table", d)):
        _check_tensor(weights[nme], dt, cfgb.num_buckets * cfgb.n_heads, nme)
    for nme in ("enc_final_scale", "dec_final_scale"):
        _check_tensor(weights[nme], dt, d.d_model, nme)
    if not ec.tied_logits:
        _check_tensor(weights["logits_w"], dt, ec.vocab * d.d_model, "logits_w")
    if len(weights["enc_layers"]) != ec.n_enc_layers or len(weights["dec_layers"]) != ec.n_dec_layers:
        raise ValueError("layer lists must hold n_enc_layers / n_dec_layers dicts")
    elw = (_Weights * ec.n_enc_layers)()
    for l, lw in enumerate(weights["enc_layers"]):
        elw[l] = _weights_struct(e, dict(lw, rel_table=weights["enc_rel_table"]))
    dlw = (_Weights * ec.n_dec_layers)()
    dxw = (_CrossWeights * ec.n_dec_layers)()
    for l, lw in enumerate(weights["dec_layers"]):
        dlw[l] = _weights_struct(d, dict(lw, rel_table=weights["dec_rel_table"]))
        dxw[l] = _cross_weights_struct(d, lw)
    p = lambda t: t.data_ptr()
    ws = _EncDecWeights(p(weights["embedding"]), p(weights["enc_rel_table"]), elw, p(weights["enc_final_scale"]),
                        p(weights["dec_rel_table"]), dlw, dxw, p(weights["dec_final_scale"]),
                        None if ec.tied_logits else p(weights["logits_w"]))
    gs_ref = None
    if want_grads:
        if grads is None:
            grads = alloc_encdec_grads(ec, weights)
        for nme in _ENCDEC_FLAT + (() if ec.tied_logits else ("logits_w",)):
            _check_tensor(grads[nme], torch.float32, weights[nme].numel(), "grad " + nme)
        elg = (_Grads * ec.n_enc_layers)()
        for l, gd in enumerate(grads["enc_layers"]):
            for nme in _block_names(e, LAYER_WEIGHT_NAMES):
                _check_tensor(gd[nme], torch.float32, weights["enc_layers"][l][nme].numel(), f"grad enc {l} {nme}")
            elg[l] = _Grads(*[(_addr(gd, nme) if nme != "rel_table" else p(grads["enc_rel_table"])) for nme in WEIGHT_NAMES])
        dlg = (_Grads * ec.n_dec_layers)()
        dxg = (_CrossGrads * ec.n_dec_layers)()
        for l, gd in enumerate(grads["dec_layers"]):
            for nme in _block_names(d, LAYER_WEIGHT_NAMES) + CROSS_WEIGHT_NAMES:
                _check_tensor(gd[nme], torch.float32, weights["dec_layers"][l][nme].numel(), f"grad dec {l} {nme}")
            dlg[l] = _Grads(*[(_addr(gd, nme) if nme != "rel_table" else p(grads["dec_rel_table"])) for nme in WEIGHT_NAMES])
            dxg[l] = _CrossGrads(*[p(gd[nme]) for nme in CROSS_WEIGHT_NAMES])
        gs = _EncDecGrads(p(grads["embedding"]), p(grads["enc_rel_table"]), elg, p(grads["enc_final_scale"]),
                          p(grads["dec_rel_table"]), dlg, dxg, p(grads["dec_final_scale"]),
                          None if ec.tied_logits else p(grads["logits_w"]))
        gs_ref = C.byref(gs)
    else:
        grads = None
    if loss is None:
        loss = torch.zeros(1, dtype=torch.float32, device=enc_tokens.device)
    if workspace is None:
        workspace = _byte_buffer(lib().t5_encdec_workspace_bytes(C.byref(cs)), enc_tokens.device)
    rc = lib().t5_encdec_loss_and_grad(C.byref(cs), _ptr(enc_tokens), _ptr(dec_tokens), _ptr(targets), C.byref(ws),
                                       _ptr(loss), gs_ref, int(bool(accumulate)), _ptr(workspace), workspace.numel(),
                                       _stream())
    if rc:
        raise T5Error(rc, "t5_encdec_loss_and_grad")
    return loss, grads


def adafactor_workspace_bytes(rows: int, cols: int, factored: bool) -> int:
    return int(lib().adafactor_workspace_bytes(int(rows), int(cols), int(bool(factored))))


def adafactor_step(param, grad, *, step, lr, factored, v_row=None, v_col=None, v_full=None, decay_pow=0.8,
                   eps1=1e-30, eps2=1e-3, clip=1.0, scale_by_param=True, bf16_copy_out=None, workspace=None,
                   weight_decay=0.0):
    """In-place Adafactor update of a float32 tensor viewed as [rows, cols] (1-D tensors: rows = 1)."""
    rows, cols = (param.shape[0], param.numel() // param.shape[0]) if param.dim() >= 2 else (1, param.numel())
    _check_tensor(param, torch.float32, rows * cols, "param")
    _check_tensor(grad, torch.float32, rows * cols, "grad")
    if factored:
        _check_tensor(v_row, torch.float32, rows, "v_row")
        _check_tensor(v_col, torch.float32, cols, "v_col")
    else:
        _check_tensor(v_full, torch.float32, rows * cols, "v_full")
    if bf16_copy_out is not None:
        _check_tensor(bf16_copy_out, torch.bfloat16, rows * cols, "bf16_copy_out")
    if workspace is None:
        workspace = _byte_buffer(adafactor_workspace_bytes(rows, cols, factored), param.device)
    cfg = _AfCfg(lr, decay_pow, eps1, eps2, clip, int(bool(scale_by_param)), int(step), 0.0, float(weight_decay))
    rc = lib().adafactor_step(_ptr(param), _ptr(grad), _ptr(v_row), _ptr(v_col), _ptr(v_full), rows, cols,
                              int(bool(factored)), C.byref(cfg), _ptr(bf16_copy_out), _ptr(workspace),
                              workspace.numel(), _stream())
    if rc:
        raise T5Error(rc, "adafactor_step")
    return param


def adafactor_step_static(param, grad, *, step, lr, factored, v_row=None, v_col=None, v_full=None, decay_pow=0.8,
                          eps1=1e-30, eps2=1e-3, clip=1.0, scale_by_param=True, bf16_copy_out=None,
                          weight_decay=0.0):
    """adafactor_step through the entry point that allocates nothing: no workspace argument, the scratch is a
    fixed device array inside the library (tensors beyond its size are refused)."""
    rows, cols = (param.shape[0], param.numel() // param.shape[0]) if param.dim() >= 2 else (1, param.numel())
    _check_tensor(param, torch.float32, rows * cols, "param")
    _check_tensor(grad, torch.float32, rows * cols, "grad")
    if factored:
        _check_tensor(v_row, torch.float32, rows, "v_row")
        _check_tensor(v_col, torch.float32, cols, "v_col")
    else:
        _check_tensor(v_full, torch.float32, rows * cols, "v_full")
    if bf16_copy_out is not None:
        _check_tensor(bf16_copy_out, torch.bfloat16, rows * cols, "bf16_copy_out")
    cfg = _AfCfg(lr, decay_pow, eps1, eps2, clip, int(bool(scale_by_param)), int(step), 0.0, float(weight_decay))
    rc = lib().adafactor_step_static(_ptr(param), _ptr(grad), _ptr(v_row), _ptr(v_col), _ptr(v_full), rows, cols,
                                     int(bool(factored)), C.byref(cfg), _ptr(bf16_copy_out), _stream())
    if rc:
        raise T5Error(rc, "adafactor_step_static")
    return param


def _af_tensor_array(tensors):
    """tensors: list of dicts with param, grad, factored and v_row/v_col or v_full (+ bf16_copy_out)."""
    arr = (_AfTensor * len(tensors))()
    for i, t in enumerate(tensors):
        p = t["param"]
        rows, cols = (p.shape[0], p.numel() // p.shape[0]) if p.dim() >= 2 else (1, p.numel())
        fact = bool(t["factored"])
        _check_tensor(p, torch.float32, rows * cols, "param")
        _check_tensor(t["grad"], torch.float32, rows * cols, "grad")
        if fact:
            _check_tensor(t["v_row"], torch.float32, rows, "v_row")
            _check_tensor(t["v_col"], torch.float32, cols, "v_col")
        else:
            _check_tensor(t["v_full"], torch.float32, rows * cols, "v_full")
        lp = t.get("bf16_copy_out")
        if lp is not None:
            _check_tensor(lp, torch.bfloat16, rows * cols, "bf16_copy_out")
        mom = t.get("m")
        if mom is not None:
            _check_tensor(mom, torch.float32, rows * cols, "m")
        addr = lambda x: None if x is None else x.data_ptr()
        arr[i] = _AfTensor(addr(p), addr(t["grad"]), addr(t.get("v_row")) if fact else None,
                           addr(t.get("v_col")) if fact else None, None if fact else addr(t.get("v_full")),
                           rows, cols, int(fact), addr(lp), addr(mom))
    return arr


def adafactor_multi_workspace_bytes(tensors) -> int:
    arr = _af_tensor_array(tensors)
    return int(lib().adafactor_multi_workspace_bytes(arr, len(tensors)))


def adafactor_step_multi(tensors, *, step, lr, decay_pow=0.8, eps1=1e-30, eps2=1e-3, clip=1.0,
                         scale_by_param=True, workspace=None, beta1=0.0, weight_decay=0.0):
    """In-place Adafactor update of several float32 tensors in one sequence of launches.  beta1 > 0 adds
    momentum (each tensor dict then holds its float32 buffer "m"); weight_decay is decoupled."""
    arr = _af_tensor_array(tensors)
    if workspace is None:
        workspace = _byte_buffer(max(int(lib().adafactor_multi_workspace_bytes(arr, len(tensors))), 256),
                                 tensors[0]["param"].device)
    cfg = _AfCfg(lr, decay_pow, eps1, eps2, clip, int(bool(scale_by_param)), int(step), float(beta1),
                 float(weight_decay))
    rc = lib().adafactor_step_multi(arr, len(tensors), C.byref(cfg), _ptr(workspace), workspace.numel(), _stream())
    if rc:
        raise T5Error(rc, "adafactor_step_multi")


def t5_gemm_bf16(a: torch.Tensor, b: torch.Tensor, a_kc: bool, b_kc: bool, out: torch.Tensor | None = None):
    """C[m,n] = sum_k A(m,k) B(n,k) in float32.  a: [M,K] if a_kc else [K,M]; b: [N,K] if b_kc else [K,N]."""
    for t, nme in ((a, "a"), (b, "b")):
        _check_tensor(t, torch.bfloat16, t.numel(), nme)
    M, K = (a.shape[0], a.shape[1]) if a_kc else (a.shape[1], a.shape[0])
    N = b.shape[0] if b_kc else b.shape[1]
    if out is None:
        out = torch.empty(M, N, dtype=torch.float32, device=a.device)
    rc = lib().t5_gemm_bf16(_ptr(a), _ptr(b), _ptr(out), M, N, K, a.shape[1], b.shape[1], N, int(a_kc), int(b_kc),
                            _stream())
    if rc:
        raise T5Error(rc, "t5_gemm_bf16")
    return out


def t5_wgrad_overlap_enable(enable: bool) -> None:
    """Run the weight-gradient GEMMs of every backward pass on a second stream owned by the library."""
    rc = lib().t5_wgrad_overlap_enable(int(bool(enable)))
    if rc:
        raise T5Error(rc, "t5_wgrad_overlap_enable")


def t5_step_timing_enable(enable: bool) -> None:
    lib().t5_step_timing_enable(int(bool(enable)))


def t5_mfma_peak_probe(workgroups: int, iters: int, random_operands: bool, sink: torch.Tensor) -> float:
    """Launches the register-only MFMA loop; returns the FLOPs it performs (the caller times it)."""
    _check_tensor(sink, torch.float32, 256, "sink")
    rc = lib().t5_mfma_peak_probe(int(workgroups), int(iters), int(bool(random_operands)), _ptr(sink), _stream())
    if rc:
        raise T5Error(rc, "t5_mfma_peak_probe")
    return float(workgroups) * 4 * iters * 32 * 2.0 * 32 * 32 * 16


def t5_step_timing_read(cap: int = 64) -> dict:
    """{step name: (total ms, launches)} since timing was enabled."""
    names = (C.c_char_p * cap)()
    ms = (C.c_float * cap)()
    calls = (C.c_int * cap)()
    n = lib().t5_step_timing_read(names, ms, calls, cap)
    return {names[i].decode(): (float(ms[i]), int(calls[i])) for i in range(n)}
