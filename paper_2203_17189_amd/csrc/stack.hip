// C-ABI entry points of whole layer stacks (see include/t5mi.h): token embedding, n_layers blocks that
// share one relative-position table, final norm, logits and loss, forward and backward in one call --
// a single stack (decoder-only or encoder-style) and the encoder-decoder pair in which every decoder
// layer cross-attends to the encoder's output.
#include "block_host.h"

namespace {

constexpr int kLogitChunk = 16384;  // tokens whose logits exist at a time

// ------------------------------------------------------------------------------------------------
// One stack of identical layers.  Layer l reads x_l and writes x_{l+1} (storage type); its saved
// activations go to stash l (or to the one shared stash with remat).  The bias diagonals of the shared
// table are built once; every layer's backward adds into one ddiag buffer, folded into buckets once.
// ------------------------------------------------------------------------------------------------
struct Layers {
  const t5_block_cfg* bc = nullptr;
  Dims D;          // D.Sk > 0: decoder layers with cross-attention over an encoder output of that length
  RelposLut lut;
  int L = 0;
  int layer0 = 0;  // index of the first layer in the model's count of layers (dropout seeds)
  bool remat = false, fused = false;
  std::vector<t5_block_weights> lw;
  std::vector<t5_block_grads> lg;
  std::vector<t5_cross_weights> xw;
  std::vector<t5_cross_grads> xg;
  const void* rel_table = nullptr;
  float* d_rel_table = nullptr;
  // carved device memory
  void* xs = nullptr;
  void* stash = nullptr;
  size_t stash_each = 0;
  float *diag = nullptr, *ddiag = nullptr;
  void* block_ws = nullptr;
  void *dxa = nullptr, *dxb = nullptr;
  // Weight gradients of all layers in grouped launches after the backward sweep (see wgrads_grouped_ok):
  // every layer then keeps its own backward workspace and incoming gradient until the sweep is over.
  bool grouped = false;
  void* layer_ws = nullptr;   // L - 1 more backward workspaces (layer L-1 uses block_ws)
  size_t bwd_ws_each = 0;
  void* dx_more = nullptr;    // L - 1 more gradient buffers
  const void** ptr_tab = nullptr;

  size_t xbytes() const { return (size_t)D.T * D.d * D.es; }
  void* x_of(int l) const { return (char*)xs + (size_t)l * xbytes(); }
  void* stash_of(int l) const { return (char*)stash + (remat ? 0 : (size_t)l * stash_each); }
};

// The weight-gradient GEMMs of one layer reduce over that layer's tokens only; at 16 k tokens and less they
// are short split-k problems that leave the chip half idle.  Launched for all layers at once (same shapes,
// a pointer table per problem) they fill it without splitting.  That needs every layer's operands alive
// until the end of the sweep: its saved activations (so: no remat) and its backward workspace.
constexpr int kWgradKinds = 7;  // wo_ff, wi, wo, wqkv; decoder layers: xo, xq, xkv
GemmDesc wgrad_desc(const Dims& D, int kind, const void* A, const void* B) {
  const int T = (int)D.T, Te = (int)D.Te, nf = D.mlp == ACT_RELU ? 1 : 2;
  switch (kind) {
    case 0: return gemm1(D.F, D.d, T, A, D.F, 0, B, D.d, 0, D.ty);            // dWo_ff = a^T dy
    case 1: return gemm1(D.d, nf * D.F, T, A, D.d, 0, B, nf * D.F, 0, D.ty);  // dWi0 | dWi1 = n2^T [du | dw]
    case 2: return gemm1(D.I, D.d, T, A, D.I, 0, B, D.d, 0, D.ty);            // dWo = c^T dh
    case 3: return gemm1(D.d, 3 * D.I, T, A, D.d, 0, B, 3 * D.I, 0, D.ty);    // dWq | dWk | dWv = n1^T dqkv
    case 4: return gemm1(D.I, D.d, T, A, D.I, 0, B, D.d, 0, D.ty);            // dXo = cx^T dh2
    case 5: return gemm1(D.d, D.I, T, A, D.d, 0, B, D.I, 0, D.ty);            // dXq = nx^T dq
    default: return gemm1(D.d, 2 * D.I, Te, A, D.d, 0, B, 2 * D.I, 0, D.ty);  // dXk | dXv = enc^T [dk | dv]
  }
}
GemmEpi wgrad_epi(const Dims& D, int kind, float* o0, float* o1, float* o2) {
  const int ld = kind == 0 || kind == 2 || kind == 4 ? D.d : kind == 1 ? D.F : D.I;
  GemmEpi e = epi(EPI_SPLIT_F32, o0, ld, IN_F32);
  e.out1 = o1; e.out2 = o2; e.accumulate = 1;
  if (kind == 1 && D.mlp != ACT_RELU) e.split_n = D.F;
  if (kind == 3 || kind == 6) e.split_n = D.I;
  return e;
}
bool wgrads_grouped_ok(const Dims& D, int L, bool remat) {
  // (the reproducible mode keeps the per-layer launches: their split reductions go through the two-pass form)
  if (D.ty != IN_BF16 || remat || L < 2 || L > 256 || D.det) return false;
  alignas(16) static const long long dummy[4] = {0, 0, 0, 0};
  for (int kind = 0; kind < (D.Sk > 0 ? kWgradKinds : 4); ++kind) {
    GemmDesc g = wgrad_desc(D, kind, dummy, dummy);
    g.groups = (const void* const*)dummy; g.ngroups = L;
    if (!gemm_mfma_supported(g, wgrad_epi(D, kind, (float*)dummy, (float*)dummy, (float*)dummy))) return false;
  }
  return true;
}

void carve_layers(Carver& cv, Layers& s) {
  const Dims& D = s.D;
  s.xs = cv.take((size_t)(s.L + 1) * s.xbytes());
  s.stash_each = carve_stash(D, nullptr, nullptr);
  s.stash = cv.take(s.stash_each * (s.remat ? 1 : s.L));
  s.diag = cv.take<float>((size_t)D.H * (2 * D.S - 1) * 4);
  s.ddiag = cv.take<float>((size_t)D.H * (2 * D.S - 1) * 4);
  const size_t f = carve_fwd(D, nullptr, nullptr), b = carve_bwd(D, nullptr, nullptr);
  s.block_ws = cv.take(f > b ? f : b);
  s.dxa = cv.take(s.xbytes());
  s.dxb = cv.take(s.xbytes());
  s.grouped = wgrads_grouped_ok(D, s.L, s.remat);
  if (s.grouped) {
    s.bwd_ws_each = b;
    s.layer_ws = cv.take(b * (size_t)(s.L - 1));
    s.dx_more = cv.take(s.xbytes() * (size_t)(s.L - 1));
    s.ptr_tab = cv.take<const void*>(sizeof(void*) * kWgradKinds * GEMM_GROUP_PTRS * (size_t)s.L);
  }
}

// Copies the caller's per-layer pointer structs, pointing every layer at the stack's shared table.
int bind_layers(Layers& s, const t5_block_weights* layers, const t5_cross_weights* cross, const void* rel_table,
                const t5_block_grads* glayers, const t5_cross_grads* gcross, float* d_rel_table, bool want_grads) {
  if (!layers || !rel_table) return T5_ERR_NULL;
  const bool dec = s.D.Sk > 0;
  if (dec && !cross) return T5_ERR_NULL;
  s.rel_table = rel_table;
  s.lw.assign(layers, layers + s.L);
  for (auto& w : s.lw) {
    w.rel_table = rel_table;
    if (!weights_present(&w, s.D)) return T5_ERR_NULL;
  }
  if (dec) {
    s.xw.assign(cross, cross + s.L);
    for (auto& x : s.xw)
      if (!x.lnx_scale || !x.xq || !x.xk || !x.xv || !x.xo) return T5_ERR_NULL;
  }
  if (!want_grads) return T5_OK;
  if (!glayers || !d_rel_table || (dec && !gcross)) return T5_ERR_NULL;
  s.d_rel_table = d_rel_table;
  s.lg.assign(glayers, glayers + s.L);
  for (auto& g : s.lg) {
    g.rel_table = d_rel_table;  // never written per layer: the shared table's gradient is folded once
    if (!grads_present(&g, s.D)) return T5_ERR_NULL;
  }
  if (dec) {
    s.xg.assign(gcross, gcross + s.L);
    for (auto& x : s.xg)
      if (!x.lnx_scale || !x.xq || !x.xk || !x.xv || !x.xo) return T5_ERR_NULL;
  }
  return T5_OK;
}

// Configuration of layer l: the stack's, with the layer's own dropout seed -- the stack's plus a multiple
// of an odd 64-bit constant, so that no two layers of a model share masks.
void layer_cfg(const Layers& s, int l, t5_block_cfg* bc, Dims* D) {
  *bc = *s.bc;
  *D = s.D;
  if (s.D.drop > 0.f) {
    D->seed = s.D.seed + (uint64_t)(s.layer0 + l + 1) * 0x9E3779B97F4A7C15ull;
    bc->dropout_seed_lo = (uint32_t)D->seed;
    bc->dropout_seed_hi = (uint32_t)(D->seed >> 32);
  }
}

// In-place dropout of [rows, d] activations or gradients at one of the stack's end sites.
int end_dropout(const Dims& D, int site, void* p, int type, hipStream_t st) {
  if (D.drop > 0.f) T5_STEP("dropout_end", launch_dropout_apply(drop_site(D, site), p, p, type, D.T, D.d, st));
  return T5_OK;
}

int layer_forward(const Layers& s, int l, const void* enc_out, hipStream_t st) {
  t5_block_cfg bc;
  Dims D;
  layer_cfg(s, l, &bc, &D);
  Stash S;
  carve_stash(D, s.stash_of(l), &S);
  S.diag = s.diag;
  FwdWs FW;
  carve_fwd(D, s.block_ws, &FW);
  const bool dec = D.Sk > 0;
  if (s.fused) T5_SUB(fwd_pack_weights(D, &s.lw[l], dec ? &s.xw[l] : nullptr, FW, st));
  T5_SUB(fwd_self_attn(&bc, D, s.lut, s.x_of(l), &s.lw[l], S, FW, s.fused, st, false));
  if (dec) T5_SUB(fwd_cross_attn(&bc, D, enc_out, &s.xw[l], S, FW, s.fused, st));
  T5_SUB(fwd_mlp(&bc, D, dec ? S.h2 : S.h, &s.lw[l], S, FW, s.fused, s.x_of(l + 1), st));
  return T5_OK;
}

int layers_forward(const Layers& s, const void* enc_out, hipStream_t st) {
  T5_STEP("relpos_diag", launch_relpos_diag(s.rel_table, s.bc->dtype, s.diag, s.D.S, s.D.H, s.lut, st));
  for (int l = 0; l < s.L; ++l) T5_SUB(layer_forward(s, l, enc_out, st));
  return T5_OK;
}

// s.dxa holds the gradient of x_L on entry; *dx0 points at the gradient of x_0 on return.  Decoder
// layers add their encoder-output gradients up in denc_acc (float32 [B * Sk, d]).
int layers_backward(const Layers& s, const void* enc_out, float* denc_acc, int acc, void** dx0, hipStream_t st) {
  const Dims& D = s.D;
  const int ty = D.ty;
  const bool dec = D.Sk > 0;
  // one backward workspace, or (grouped weight gradients) one per layer; likewise the gradient buffers
  const int nws = s.grouped ? s.L : 1;
  std::vector<BwdWs> bws(nws);
  for (int i = 0; i < nws; ++i) {
    carve_bwd(D, i == 0 ? s.block_ws : (void*)((char*)s.layer_ws + (size_t)(i - 1) * s.bwd_ws_each), &bws[i]);
    bws[i].ddiag = s.ddiag;
    bws[i].defer_wgrad = s.grouped;
    if (!s.grouped) bws[i].fork = fork_begin(st, D.drop == 0.f && !D.det);
  }
  const int nring = s.grouped ? s.L + 1 : 2;
  auto ring = [&](int i) -> void* {
    const int q = i % nring;
    return q == 0 ? s.dxa : q == 1 ? s.dxb : (void*)((char*)s.dx_more + (size_t)(q - 2) * s.xbytes());
  };
  {
    ZeroList z;
    std::memset(&z, 0, sizeof(z));
    z.p[0] = s.ddiag; z.n[0] = (int64_t)D.H * (2 * D.S - 1); z.count = 1;
    T5_STEP("zero_grads", launch_zero_f32(z, st));
  }
  const AttnDims ad = self_dims(s.bc, D);
  const int far = s.lut.n_thr > 0 ? s.lut.thr[s.lut.n_thr - 1] : s.lut.max_exact;
  const bool attn_mfma = ty == IN_BF16 && attn_mfma_supported(ad) && attn_bwd_mfma_fits(ad, far);
  for (int l = s.L - 1; l >= 0; --l) {
    const int n = s.L - 1 - l;  // layers processed so far
    BwdWs& BW = bws[s.grouped ? n : 0];
    void* dy = ring(n);
    void* dx = ring(n + 1);
    ForkGuard guard(BW.fork);
    if (s.remat) T5_SUB(layer_forward(s, l, enc_out, st));  // rebuilds layer l's saved activations
    t5_block_cfg bc;
    Dims D;  // this layer's (its dropout seed differs from the stack's)
    layer_cfg(s, l, &bc, &D);
    Stash S;
    carve_stash(D, s.stash_of(l), &S);
    S.diag = s.diag;
    T5_SUB(bwd_zero(D, &s.lg[l], dec ? &s.xg[l] : nullptr, nullptr, acc != 0, st));
    T5_SUB(bwd_mlp(D, dy, dec ? S.h2 : S.h, &s.lw[l], S, BW, &s.lg[l], acc, st));
    if (dec) {
      // the first layer processed stores its denc, the others add theirs to it
      T5_SUB(bwd_cross_attn(&bc, D, enc_out, &s.xw[l], S, BW, denc_acc, &s.xg[l], acc, st, true, l != s.L - 1));
      T5_SUB(bwd_self_attn(&bc, D, s.lut, s.x_of(l), BW.dh1, BW.dh1_lp, &s.lw[l], S, BW, attn_mfma, far, dx,
                           &s.lg[l], acc, st, false));
    } else {
      T5_SUB(bwd_self_attn(&bc, D, s.lut, s.x_of(l), BW.dh, BW.dh_lp, &s.lw[l], S, BW, attn_mfma, far, dx,
                           &s.lg[l], acc, st, false));
    }
    // the next layer rewrites the workspace (and, with remat, the stash) the side GEMMs read
    T5_TRY(guard.join());
  }
  if (s.grouped) {
    // one launch per kind of weight over all layers: problem n is layer L-1-n
    std::vector<const void*> tab((size_t)kWgradKinds * s.L * GEMM_GROUP_PTRS, nullptr);
    const int kinds = dec ? kWgradKinds : 4;
    for (int n = 0; n < s.L; ++n) {
      const int l = s.L - 1 - n;
      Stash S;
      carve_stash(D, s.stash_of(l), &S);
      const BwdWs& W = bws[n];
      const t5_block_grads& g = s.lg[l];
      auto put = [&](int kind, const void* A, const void* B, float* o0, float* o1, float* o2) {
        const void** t = &tab[((size_t)kind * s.L + n) * GEMM_GROUP_PTRS];
        t[0] = A; t[1] = B; t[2] = o0; t[3] = o1; t[4] = o2;
      };
      // with dropout the GEMMs of a dropped sublayer output read its masked gradient copy
      const bool drop = D.drop > 0.f;
      put(0, S.a, drop ? W.dmask : ring(n), g.wo_ff, nullptr, nullptr);
      put(1, S.n2, W.duw, g.wi0, D.mlp == ACT_RELU ? nullptr : g.wi1, nullptr);
      put(2, S.c, drop ? W.dmask_a : (dec ? W.dh1_lp : W.dh_lp), g.wo, nullptr, nullptr);
      put(3, S.n1, W.dqkv, g.wq, g.wk, g.wv);
      if (dec) {
        const t5_cross_grads& x = s.xg[l];
        put(4, S.cx, drop ? W.dmask_x : W.dh_lp, x.xo, nullptr, nullptr);
        put(5, S.nx, W.dqx, x.xq, nullptr, nullptr);
        put(6, enc_out, W.dkvx, x.xk, x.xv, nullptr);
      }
    }
    T5_STEP("wgrad_table", launch_fill_ptrs(tab.data(), kinds * s.L * GEMM_GROUP_PTRS, s.ptr_tab, st));
    static const char* const names[kWgradKinds] = {"gemm_dwo_ff", "gemm_dwi", "gemm_dwo", "gemm_dwqkv",
                                                   "gemm_dxo", "gemm_dxq", "gemm_dxkv"};
    for (int kind = 0; kind < kinds; ++kind) {
      const void** t = &tab[(size_t)kind * s.L * GEMM_GROUP_PTRS];
      GemmDesc g = wgrad_desc(D, kind, t[0], t[1]);
      g.groups = s.ptr_tab + (size_t)kind * s.L * GEMM_GROUP_PTRS;
      g.ngroups = s.L;
      const GemmEpi e = wgrad_epi(D, kind, (float*)t[2], (float*)t[3], (float*)t[4]);
      if (!gemm_mfma_supported(g, e)) return T5_ERR_UNSUPPORTED;  // checked for the shapes when the plan was made
      T5_STEP(names[kind], launch_gemm_mfma(g, e, st));
    }
  }
  T5_STEP("relpos_diag_bwd",
          launch_relpos_diag_bwd(s.ddiag, s.d_rel_table, D.S, D.H, s.bc->num_buckets, s.lut, acc, st));
  *dx0 = ring(s.L);
  return T5_OK;
}

// ------------------------------------------------------------------------------------------------
// Head: final norm, logits a chunk of tokens at a time, loss and its gradient in place, the two
// gradient GEMMs.  Leaves the gradient of the stack's last output in `dx_out` (storage type).
// ------------------------------------------------------------------------------------------------
struct Head {
  int V = 0, chunk = 0;
  bool tied = false;
  float z_loss = 0.f;
  int drop_site_final = DROP_FINAL;  // dropout site of the final norm's output
  const void *embedding = nullptr, *final_scale = nullptr, *logits_w = nullptr;
  float *d_embedding = nullptr, *d_final_scale = nullptr, *d_logits_w = nullptr;
  void *nf = nullptr, *logits = nullptr, *wout_t = nullptr, *scale_s = nullptr;
  float *rf = nullptr, *loss_rows = nullptr, *n_valid = nullptr, *dnf = nullptr, *dg_tmp = nullptr,
        *dg_partial = nullptr;
  float* wg_partials = nullptr;  // reproducible mode: partial sums of the output-matrix gradient's k-slices
};

// The gradient GEMM of the output matrix (or of the tied embedding) for one chunk of tokens.
void head_wgrad_gemm(const Head& h, const Dims& D, int tc, const void* nf_c, GemmDesc& g, GemmEpi& e) {
  if (h.tied) {  // dE += dlogits^T nf'
    g = gemm1(h.V, D.d, tc, h.logits, h.V, 0, nf_c, D.d, 0, D.ty);
    e = epi(EPI_SPLIT_F32, h.d_embedding, D.d, IN_F32);
  } else {  // dWout += nf^T dlogits
    g = gemm1(D.d, h.V, tc, nf_c, D.d, 0, h.logits, h.V, 0, D.ty);
    e = epi(EPI_SPLIT_F32, h.d_logits_w, h.V, IN_F32);
  }
  e.accumulate = 1;
  e.aux0 = h.wg_partials;  // null unless the reproducible mode carved it
}

void carve_head(Carver& cv, Head& h, const Dims& D) {
  h.nf = cv.take((size_t)D.T * D.d * D.es);
  h.logits = cv.take((size_t)h.chunk * h.V * D.es);
  h.wout_t = cv.take((size_t)h.V * D.d * D.es);
  h.scale_s = cv.take((size_t)D.d * D.es);
  h.rf = cv.take<float>(D.T * 4);
  h.loss_rows = cv.take<float>(D.T * 4);
  h.n_valid = cv.take<float>(256);
  h.dnf = cv.take<float>((size_t)D.T * D.d * 4);
  h.dg_tmp = cv.take<float>((size_t)D.d * 4);
  h.dg_partial = cv.take<float>((size_t)rmsnorm_bwd_partial_rows((int)D.T) * D.d * 4);
  h.wg_partials = nullptr;
  if (D.det && D.ty == IN_BF16) {
    GemmDesc g;
    GemmEpi e;
    head_wgrad_gemm(h, D, h.chunk, h.nf, g, e);
    h.wg_partials = cv.take<float>(gemm_split_partials_bytes(g, e));
  }
}

int head_loss_and_grad(const Head& h, const Dims& D, float rms_eps, const void* x_last, const int32_t* targets,
                       float* loss, bool want_grads, int acc, void* dx_out, hipStream_t st) {
  const int T = (int)D.T, ty = D.ty, V = h.V;
  const size_t es = D.es;
  // tied logits: the factor d_model^-1/2 rides on the final norm's scale, nf' = RMSNorm(x; s gf) = s nf,
  // so logits = nf' E^T, dE += dlogits^T nf' and the norm backward returns d/d(s gf), scaled back below
  const float s_tied = h.tied ? 1.f / std::sqrt((float)D.d) : 1.f;
  const void* gf = h.final_scale;
  if (h.tied) {
    T5_STEP("scale_vec", launch_scale_vec(h.scale_s, h.final_scale, s_tied, D.d, ty, st));
    gf = h.scale_s;
  }
  T5_STEP("rmsnorm_fwd", launch_rmsnorm_fwd(x_last, ty, gf, h.nf, ty, h.rf, T, D.d, rms_eps, st));
  T5_SUB(end_dropout(D, h.drop_site_final, h.nf, ty, st));  // the logits (and dW) see the dropped norm output
  // The MFMA GEMMs want the contraction index contiguous in both operands.  logits = nf W contracts over
  // d_model: E [V, d] has it contiguous, Wout [d, V] is transposed once per step.  dnf = dlogits W^T
  // contracts over the vocabulary: Wout has it contiguous, E is transposed once per step.
  const bool head_mfma = ty == IN_BF16 && D.d % 64 == 0 && V % 64 == 0;
  if (head_mfma && (!h.tied || want_grads)) {
    PackJobs pj;
    std::memset(&pj, 0, sizeof(pj));
    if (h.tied) pj.j[0] = PackJob{{h.embedding, nullptr, nullptr}, 1, V, D.d, 0, h.wout_t};   // -> [d, V]
    else pj.j[0] = PackJob{{h.logits_w, nullptr, nullptr}, 1, D.d, V, 0, h.wout_t};            // -> [V, d]
    pj.count = 1;
    T5_STEP("pack_logits_w", launch_pack_transpose_multi(pj, st));
  }
  T5_STEP("xent_count", launch_xent_count(targets, D.T, V, h.n_valid, st));
  for (int64_t t0 = 0; t0 < D.T; t0 += h.chunk) {
    const int tc = (int)std::min<int64_t>(h.chunk, D.T - t0);
    const void* nf_c = at((const void*)h.nf, (size_t)t0 * D.d, es);
    {  // logits = nf W
      GemmDesc g;
      if (h.tied) g = gemm1(tc, V, D.d, nf_c, D.d, 1, h.embedding, D.d, 1, ty);
      else if (head_mfma) g = gemm1(tc, V, D.d, nf_c, D.d, 1, h.wout_t, D.d, 1, ty);
      else g = gemm1(tc, V, D.d, nf_c, D.d, 1, h.logits_w, V, 0, ty);
      T5_STEP("gemm_logits", run_gemm(g, epi(EPI_STORE, h.logits, V, ty), st));
    }
    T5_STEP("xent_rows", launch_xent_rows(h.logits, ty, targets + t0, tc, V, V, h.z_loss, h.n_valid,
                                          h.loss_rows + t0, want_grads ? 1 : 0, st));
    if (!want_grads) continue;
    {  // dnf = dlogits W^T
      GemmDesc g;
      if (!h.tied) g = gemm1(tc, D.d, V, h.logits, V, 1, h.logits_w, V, 1, ty);
      else if (head_mfma) g = gemm1(tc, D.d, V, h.logits, V, 1, h.wout_t, V, 1, ty);
      else g = gemm1(tc, D.d, V, h.logits, V, 1, h.embedding, D.d, 0, ty);
      T5_STEP("gemm_dnf", run_gemm(g, epi(EPI_STORE, h.dnf + (size_t)t0 * D.d, D.d, IN_F32), st));
    }
    {
      GemmDesc g;
      GemmEpi e;
      head_wgrad_gemm(h, D, tc, nf_c, g, e);
      T5_STEP("gemm_dlogits_w", run_gemm(g, e, st));
    }
  }
  T5_STEP("loss_reduce", launch_loss_reduce(h.loss_rows, D.T, h.n_valid, loss, st));
  if (!want_grads) return T5_OK;
  // gradient of the stack's last output through the final norm (no residual term)
  float* dg = h.tied ? h.dg_tmp : h.d_final_scale;
  T5_SUB(end_dropout(D, h.drop_site_final, h.dnf, IN_F32, st));
  T5_STEP("rmsnorm_bwd", launch_rmsnorm_bwd(x_last, ty, gf, ty, h.rf, h.dnf, nullptr, IN_F32,
                                            ty == IN_F32 ? (float*)dx_out : nullptr, ty == IN_BF16 ? dx_out : nullptr,
                                            ty, dg, h.dg_partial, h.tied ? 0 : acc, T, D.d, st));
  if (h.tied) T5_STEP("axpy", launch_axpy_f32(h.d_final_scale, h.dg_tmp, s_tied, D.d, acc, st));
  return T5_OK;
}

int validate_ends(int n_layers, int vocab, float z_loss) {
  if (n_layers < 1 || vocab < 2 || !(z_loss >= 0.f) || !std::isfinite(z_loss)) return T5_ERR_SHAPE;
  if (n_layers > 1024 || vocab > (1 << 22)) return T5_ERR_UNSUPPORTED;
  return T5_OK;
}

// Clears the embedding and output-matrix gradients that the kernels add into.
int zero_end_grads(float* d_embedding, float* d_logits_w, int V, int d, hipStream_t st) {
  ZeroList z;
  std::memset(&z, 0, sizeof(z));
  z.p[z.count] = d_embedding; z.n[z.count] = (int64_t)V * d; ++z.count;
  if (d_logits_w) { z.p[z.count] = d_logits_w; z.n[z.count] = (int64_t)d * V; ++z.count; }
  T5_STEP("zero_grads", launch_zero_f32(z, st));
  return T5_OK;
}

// ---- single stack
struct StackPlan {
  Layers S;
  Head H;
};
int plan_stack(const t5_stack_cfg* c, StackPlan* p) {
  if (!c) return T5_ERR_NULL;
  int rc = validate_cfg(&c->block, &p->S.D, &p->S.lut);
  if (rc != T5_OK) return rc;
  if ((rc = validate_ends(c->n_layers, c->vocab, c->z_loss)) != T5_OK) return rc;
  p->S.bc = &c->block; p->S.L = c->n_layers; p->S.remat = c->remat != 0; p->S.fused = fused_fwd_ok(p->S.D);
  p->H.V = c->vocab; p->H.tied = c->tied_logits != 0; p->H.z_loss = c->z_loss;
  p->H.chunk = p->S.D.T < kLogitChunk ? (int)p->S.D.T : kLogitChunk;
  return T5_OK;
}
size_t carve_stack(StackPlan& p, void* base) {
  Carver cv(base);
  carve_layers(cv, p.S);
  carve_head(cv, p.H, p.S.D);
  return cv.off;
}

// ---- encoder-decoder pair
struct EncDecPlan {
  Layers E, Dc;
  Head H;
  void* enc_out = nullptr;     // [B * S_enc, d] storage type: RMSNorm of the encoder's last output
  float* enc_rf = nullptr;     // [B * S_enc]
  float* denc = nullptr;       // [B * S_enc, d] float32: sum of the decoder layers' encoder-output gradients
  float* enc_dg_partial = nullptr;
  t5_block_cfg dec_bc;
};
int plan_encdec(const t5_encdec_cfg* c, EncDecPlan* p) {
  if (!c) return T5_ERR_NULL;
  const t5_block_cfg& e = c->enc_block;
  const t5_block_cfg& d = c->dec_block;
  if (e.causal != 0 || d.causal == 0) return T5_ERR_SHAPE;  // bidirectional encoder, causal decoder
  if (e.batch != d.batch || e.d_model != d.d_model || e.dtype != d.dtype) return T5_ERR_SHAPE;
  int rc = validate_cfg(&e, &p->E.D, &p->E.lut);
  if (rc != T5_OK) return rc;
  if ((rc = validate_cfg(&d, &p->Dc.D, &p->Dc.lut, e.seq)) != T5_OK) return rc;
  if ((rc = validate_ends(c->n_enc_layers, c->vocab, c->z_loss)) != T5_OK) return rc;
  if ((rc = validate_ends(c->n_dec_layers, c->vocab, c->z_loss)) != T5_OK) return rc;
  p->E.bc = &c->enc_block; p->E.L = c->n_enc_layers; p->E.remat = c->remat != 0; p->E.fused = fused_fwd_ok(p->E.D);
  p->Dc.layer0 = c->n_enc_layers;  // the decoder's layers count on from the encoder's
  p->H.drop_site_final = DROP_DEC_FINAL;
  p->Dc.bc = &c->dec_block; p->Dc.L = c->n_dec_layers; p->Dc.remat = c->remat != 0; p->Dc.fused = fused_fwd_ok(p->Dc.D);
  p->H.V = c->vocab; p->H.tied = c->tied_logits != 0; p->H.z_loss = c->z_loss;
  p->H.chunk = p->Dc.D.T < kLogitChunk ? (int)p->Dc.D.T : kLogitChunk;
  return T5_OK;
}
size_t carve_encdec(EncDecPlan& p, void* base) {
  Carver cv(base);
  carve_layers(cv, p.E);
  carve_layers(cv, p.Dc);
  carve_head(cv, p.H, p.Dc.D);
  const Dims& E = p.E.D;
  p.enc_out = cv.take((size_t)E.T * E.d * E.es);
  p.enc_rf = cv.take<float>(E.T * 4);
  p.denc = cv.take<float>((size_t)E.T * E.d * 4);
  p.enc_dg_partial = cv.take<float>((size_t)rmsnorm_bwd_partial_rows((int)E.T) * E.d * 4);
  return cv.off;
}

}  // namespace

extern "C" {

size_t t5_stack_workspace_bytes(const t5_stack_cfg* cfg) {
  StackPlan p;
  if (plan_stack(cfg, &p) != T5_OK) return 0;
  return carve_stack(p, nullptr);
}

int t5_stack_loss_and_grad(const t5_stack_cfg* cfg, const int32_t* tokens, const int32_t* targets,
                           const t5_stack_weights* w, float* loss, const t5_stack_grads* grads, int accumulate,
                           void* workspace, size_t workspace_bytes, void* stream) {
  StackPlan p;
  int rc = plan_stack(cfg, &p);
  if (rc != T5_OK) return rc;
  if (!tokens || !targets || !w || !loss || !workspace) return T5_ERR_NULL;
  if (!w->embedding || !w->final_scale || (!p.H.tied && !w->logits_w)) return T5_ERR_NULL;
  if (grads && (!grads->embedding || !grads->final_scale || (!p.H.tied && !grads->logits_w))) return T5_ERR_NULL;
  rc = bind_layers(p.S, w->layers, nullptr, w->rel_table, grads ? grads->layers : nullptr, nullptr,
                   grads ? grads->rel_table : nullptr, grads != nullptr);
  if (rc != T5_OK) return rc;
  if (workspace_bytes < carve_stack(p, nullptr)) return T5_ERR_WORKSPACE;
  carve_stack(p, workspace);
  hipStream_t st = (hipStream_t)stream;
  const Dims& D = p.S.D;
  const int acc = accumulate ? 1 : 0, V = p.H.V;
  p.H.embedding = w->embedding; p.H.final_scale = w->final_scale; p.H.logits_w = w->logits_w;
  if (grads) {
    p.H.d_embedding = grads->embedding; p.H.d_final_scale = grads->final_scale;
    p.H.d_logits_w = p.H.tied ? nullptr : grads->logits_w;
  }

  T5_STEP("embed_fwd", launch_embed_fwd(tokens, w->embedding, p.S.x_of(0), D.ty, D.T, D.d, V, st));
  T5_SUB(end_dropout(D, DROP_EMBED, p.S.x_of(0), D.ty, st));
  T5_SUB(layers_forward(p.S, nullptr, st));
  if (grads && !acc) T5_SUB(zero_end_grads(grads->embedding, p.H.d_logits_w, V, D.d, st));
  T5_SUB(head_loss_and_grad(p.H, D, cfg->block.rms_eps, p.S.x_of(p.S.L), targets, loss, grads != nullptr, acc,
                            p.S.dxa, st));
  if (!grads) return T5_OK;
  void* dx0 = nullptr;
  T5_SUB(layers_backward(p.S, nullptr, nullptr, acc, &dx0, st));
  T5_SUB(end_dropout(D, DROP_EMBED, dx0, D.ty, st));
  T5_STEP("embed_bwd", launch_embed_bwd(tokens, dx0, D.ty, grads->embedding, D.T, D.d, V, D.det, st));
  return T5_OK;
}

size_t t5_encdec_workspace_bytes(const t5_encdec_cfg* cfg) {
  EncDecPlan p;
  if (plan_encdec(cfg, &p) != T5_OK) return 0;
  return carve_encdec(p, nullptr);
}

int t5_encdec_loss_and_grad(const t5_encdec_cfg* cfg, const int32_t* enc_tokens, const int32_t* dec_tokens,
                            const int32_t* targets, const t5_encdec_weights* w, float* loss,
                            const t5_encdec_grads* grads, int accumulate, void* workspace, size_t workspace_bytes,
                            void* stream) {
  EncDecPlan p;
  int rc = plan_encdec(cfg, &p);
  if (rc != T5_OK) return rc;
  if (!enc_tokens || !dec_tokens || !targets || !w || !loss || !workspace) return T5_ERR_NULL;
  if (!w->embedding || !w->enc_final_scale || !w->dec_final_scale || (!p.H.tied && !w->logits_w)) return T5_ERR_NULL;
  if (grads && (!grads->embedding || !grads->enc_final_scale || !grads->dec_final_scale ||
                (!p.H.tied && !grads->logits_w)))
    return T5_ERR_NULL;
  rc = bind_layers(p.E, w->enc_layers, nullptr, w->enc_rel_table, grads ? grads->enc_layers : nullptr, nullptr,
                   grads ? grads->enc_rel_table : nullptr, grads != nullptr);
  if (rc != T5_OK) return rc;
  rc = bind_layers(p.Dc, w->dec_layers, w->dec_cross, w->dec_rel_table, grads ? grads->dec_layers : nullptr,
                   grads ? grads->dec_cross : nullptr, grads ? grads->dec_rel_table : nullptr, grads != nullptr);
  if (rc != T5_OK) return rc;
  if (workspace_bytes < carve_encdec(p, nullptr)) return T5_ERR_WORKSPACE;
  carve_encdec(p, workspace);
  hipStream_t st = (hipStream_t)stream;
  const Dims& E = p.E.D;
  const Dims& D = p.Dc.D;
  const int ty = D.ty, acc = accumulate ? 1 : 0, V = p.H.V;
  p.H.embedding = w->embedding; p.H.final_scale = w->dec_final_scale; p.H.logits_w = w->logits_w;
  if (grads) {
    p.H.d_embedding = grads->embedding; p.H.d_final_scale = grads->dec_final_scale;
    p.H.d_logits_w = p.H.tied ? nullptr : grads->logits_w;
  }

  // encoder: embedding, layers, final norm -> enc_out
  T5_STEP("embed_fwd", launch_embed_fwd(enc_tokens, w->embedding, p.E.x_of(0), ty, E.T, E.d, V, st));
  T5_SUB(end_dropout(E, DROP_EMBED, p.E.x_of(0), ty, st));
  T5_SUB(layers_forward(p.E, nullptr, st));
  T5_STEP("rmsnorm_fwd", launch_rmsnorm_fwd(p.E.x_of(p.E.L), ty, w->enc_final_scale, p.enc_out, ty, p.enc_rf, (int)E.T,
                                            E.d, cfg->enc_block.rms_eps, st));
  T5_SUB(end_dropout(E, DROP_FINAL, p.enc_out, ty, st));
  // decoder: embedding, layers cross-attending to enc_out, head
  T5_STEP("embed_fwd", launch_embed_fwd(dec_tokens, w->embedding, p.Dc.x_of(0), ty, D.T, D.d, V, st));
  T5_SUB(end_dropout(D, DROP_DEC_EMBED, p.Dc.x_of(0), ty, st));
  T5_SUB(layers_forward(p.Dc, p.enc_out, st));
  if (grads && !acc) T5_SUB(zero_end_grads(grads->embedding, p.H.d_logits_w, V, D.d, st));
  T5_SUB(head_loss_and_grad(p.H, D, cfg->dec_block.rms_eps, p.Dc.x_of(p.Dc.L), targets, loss, grads != nullptr, acc,
                            p.Dc.dxa, st));
  if (!grads) return T5_OK;
  void* dx0 = nullptr;
  T5_SUB(layers_backward(p.Dc, p.enc_out, p.denc, acc, &dx0, st));
  T5_SUB(end_dropout(D, DROP_DEC_EMBED, dx0, ty, st));
  T5_STEP("embed_bwd", launch_embed_bwd(dec_tokens, dx0, ty, grads->embedding, D.T, D.d, V, D.det, st));
  T5_SUB(end_dropout(E, DROP_FINAL, p.denc, IN_F32, st));
  // encoder: final norm backward (no residual term), layers, embedding
  T5_STEP("rmsnorm_bwd", launch_rmsnorm_bwd(p.E.x_of(p.E.L), ty, w->enc_final_scale, ty, p.enc_rf, p.denc, nullptr,
                                            IN_F32, ty == IN_F32 ? (float*)p.E.dxa : nullptr,
                                            ty == IN_BF16 ? p.E.dxa : nullptr, ty, grads->enc_final_scale,
                                            p.enc_dg_partial, acc, (int)E.T, E.d, st));
  T5_SUB(layers_backward(p.E, nullptr, nullptr, acc, &dx0, st));
  T5_SUB(end_dropout(E, DROP_EMBED, dx0, ty, st));
  T5_STEP("embed_bwd", launch_embed_bwd(enc_tokens, dx0, ty, grads->embedding, E.T, E.d, V, E.det, st));
  return T5_OK;
}

}  // extern "C"
