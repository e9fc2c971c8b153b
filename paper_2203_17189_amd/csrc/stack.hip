// C-ABI entry points of the layer stack: embedding, n_layers blocks that share one relative-position
// table, final norm, logits and loss, forward and backward in one call (see include/t5mi.h).
#include "block_host.h"

namespace {

constexpr int kLogitChunk = 8192;  // tokens whose logits exist at a time

struct StackDims {
  Dims D;
  int L, V;
  int chunk;  // tokens per logits chunk
  bool tied, remat;
};

int validate_stack(const t5_stack_cfg* c, StackDims* o, RelposLut* lut) {
  if (!c) return T5_ERR_NULL;
  StackDims sd;
  const int rc = validate_cfg(&c->block, &sd.D, lut);
  if (rc != T5_OK) return rc;
  if (c->n_layers < 1 || c->vocab < 2 || !(c->z_loss >= 0.f) || !std::isfinite(c->z_loss)) return T5_ERR_SHAPE;
  if (c->n_layers > 1024 || c->vocab > (1 << 22)) return T5_ERR_UNSUPPORTED;
  sd.L = c->n_layers; sd.V = c->vocab;
  sd.chunk = sd.D.T < kLogitChunk ? (int)sd.D.T : kLogitChunk;
  sd.tied = c->tied_logits != 0; sd.remat = c->remat != 0;
  if (o) *o = sd;
  return T5_OK;
}

struct StackWs {
  void* xs;           // [L + 1][T, d] storage type: layer inputs, xs[L] = output of the last layer
  void* stash;        // per-layer saved activations: L of them, or one with remat
  size_t stash_each;
  float *diag, *ddiag;  // shared bias diagonals and their gradient [H, 2S-1]
  void* block_ws;     // workspace of the block's forward / backward
  size_t block_ws_bytes;
  void *nf, *logits, *wout_t, *scale_s, *dxa, *dxb;
  float *rf, *loss_rows, *n_valid, *dnf, *dg_tmp;
};
size_t carve_stack(const StackDims& sd, void* base, StackWs* w) {
  const Dims& D = sd.D;
  Carver cv(base);
  StackWs t;
  std::memset(&t, 0, sizeof(t));
  t.xs = cv.take((size_t)(sd.L + 1) * D.T * D.d * D.es);
  t.stash_each = carve_stash(D, nullptr, nullptr);
  t.stash = cv.take(t.stash_each * (sd.remat ? 1 : sd.L));
  t.diag = cv.take<float>((size_t)D.H * (2 * D.S - 1) * 4);
  t.ddiag = cv.take<float>((size_t)D.H * (2 * D.S - 1) * 4);
  const size_t f = carve_fwd(D, nullptr, nullptr), b = carve_bwd(D, nullptr, nullptr);
  t.block_ws_bytes = f > b ? f : b;
  t.block_ws = cv.take(t.block_ws_bytes);
  t.nf = cv.take((size_t)D.T * D.d * D.es);
  t.logits = cv.take((size_t)sd.chunk * sd.V * D.es);
  t.wout_t = cv.take((size_t)sd.V * D.d * D.es);
  t.scale_s = cv.take((size_t)D.d * D.es);
  t.dxa = cv.take((size_t)D.T * D.d * D.es);
  t.dxb = cv.take((size_t)D.T * D.d * D.es);
  t.rf = cv.take<float>(D.T * 4);
  t.loss_rows = cv.take<float>(D.T * 4);
  t.n_valid = cv.take<float>(256);
  t.dnf = cv.take<float>((size_t)D.T * D.d * 4);
  t.dg_tmp = cv.take<float>((size_t)D.d * 4);
  if (w) *w = t;
  return cv.off;
}

}  // namespace

extern "C" {

size_t t5_stack_workspace_bytes(const t5_stack_cfg* cfg) {
  StackDims sd;
  if (validate_stack(cfg, &sd, nullptr) != T5_OK) return 0;
  return carve_stack(sd, nullptr, nullptr);
}

int t5_stack_loss_and_grad(const t5_stack_cfg* cfg, const int32_t* tokens, const int32_t* targets,
                           const t5_stack_weights* w, float* loss, const t5_stack_grads* grads, int accumulate,
                           void* workspace, size_t workspace_bytes, void* stream) {
  StackDims sd;
  RelposLut lut;
  const int rc = validate_stack(cfg, &sd, &lut);
  if (rc != T5_OK) return rc;
  const Dims& D = sd.D;
  const t5_block_cfg* bc = &cfg->block;
  if (!tokens || !targets || !w || !loss || !workspace) return T5_ERR_NULL;
  if (!w->embedding || !w->rel_table || !w->layers || !w->final_scale || (!sd.tied && !w->logits_w))
    return T5_ERR_NULL;
  std::vector<t5_block_weights> lw(sd.L);
  for (int l = 0; l < sd.L; ++l) {
    lw[l] = w->layers[l];
    lw[l].rel_table = w->rel_table;
    if (!weights_present(&lw[l])) return T5_ERR_NULL;
  }
  std::vector<t5_block_grads> lg(sd.L);
  if (grads) {
    if (!grads->embedding || !grads->rel_table || !grads->layers || !grads->final_scale ||
        (!sd.tied && !grads->logits_w))
      return T5_ERR_NULL;
    for (int l = 0; l < sd.L; ++l) {
      lg[l] = grads->layers[l];
      lg[l].rel_table = grads->rel_table;  // never written per layer (the shared table is folded once)
      if (!grads_present(&lg[l])) return T5_ERR_NULL;
    }
  }
  if (workspace_bytes < carve_stack(sd, nullptr, nullptr)) return T5_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  StackWs K;
  carve_stack(sd, workspace, &K);
  const int T = (int)D.T, ty = D.ty, acc = accumulate ? 1 : 0, V = sd.V;
  const size_t es = D.es;
  const size_t xbytes = (size_t)D.T * D.d * es;
  auto x_of = [&](int l) { return (void*)((char*)K.xs + (size_t)l * xbytes); };
  auto stash_of = [&](int l) { return (void*)((char*)K.stash + (sd.remat ? 0 : (size_t)l * K.stash_each)); };
  const bool fused = fused_fwd_ok(D);
  FwdWs FW;
  carve_fwd(D, K.block_ws, &FW);

  // ---------------------------------------------------------------- forward sweep
  T5_STEP("embed_fwd", launch_embed_fwd(tokens, w->embedding, x_of(0), ty, D.T, D.d, V, st));
  T5_STEP("relpos_diag", launch_relpos_diag(w->rel_table, bc->dtype, K.diag, D.S, D.H, lut, st));
  auto layer_fwd = [&](int l) -> int {
    Stash S;
    carve_stash(D, stash_of(l), &S);
    S.diag = K.diag;
    if (fused) T5_SUB(fwd_pack_weights(D, &lw[l], nullptr, FW, st));
    T5_SUB(fwd_self_attn(bc, D, lut, x_of(l), &lw[l], S, FW, fused, st, false));
    T5_SUB(fwd_mlp(bc, D, S.h, &lw[l], S, FW, fused, x_of(l + 1), st));
    return T5_OK;
  };
  for (int l = 0; l < sd.L; ++l) T5_SUB(layer_fwd(l));

  // ---------------------------------------------------------------- head: final norm, logits, loss
  // tied logits: the factor d_model^-1/2 rides on the final norm's scale, nf' = RMSNorm(x; s gf) = s nf,
  // so logits = nf' E^T, dE += dlogits^T nf' and the norm backward returns d/d(s gf), scaled back below
  const float s_tied = sd.tied ? 1.f / std::sqrt((float)D.d) : 1.f;
  const void* gf = w->final_scale;
  if (sd.tied) {
    T5_STEP("scale_vec", launch_scale_vec(K.scale_s, w->final_scale, s_tied, D.d, ty, st));
    gf = K.scale_s;
  }
  T5_STEP("rmsnorm_fwd", launch_rmsnorm_fwd(x_of(sd.L), ty, gf, K.nf, ty, K.rf, T, D.d, bc->rms_eps, st));
  // The MFMA GEMMs want the contraction index contiguous in both operands.  logits = nf W contracts over
  // d_model: E [V, d] has it contiguous, Wout [d, V] is transposed once per step.  dnf = dlogits W^T
  // contracts over the vocabulary: Wout has it contiguous, E is transposed once per step.
  const bool head_mfma = ty == IN_BF16 && D.d % 64 == 0 && V % 64 == 0;
  if (head_mfma) {
    PackJobs pj;
    std::memset(&pj, 0, sizeof(pj));
    if (sd.tied) pj.j[0] = PackJob{{w->embedding, nullptr, nullptr}, 1, V, D.d, 0, K.wout_t};   // -> [d, V]
    else pj.j[0] = PackJob{{w->logits_w, nullptr, nullptr}, 1, D.d, V, 0, K.wout_t};             // -> [V, d]
    pj.count = 1;
    if (!sd.tied || grads) T5_STEP("pack_logits_w", launch_pack_transpose_multi(pj, st));
  }
  T5_STEP("xent_count", launch_xent_count(targets, D.T, V, K.n_valid, st));
  if (grads && !acc) {
    ZeroList z;
    std::memset(&z, 0, sizeof(z));
    z.p[z.count] = grads->embedding; z.n[z.count] = (int64_t)V * D.d; ++z.count;
    if (!sd.tied) { z.p[z.count] = grads->logits_w; z.n[z.count] = (int64_t)D.d * V; ++z.count; }
    T5_STEP("zero_grads", launch_zero_f32(z, st));
  }
  for (int64_t t0 = 0; t0 < D.T; t0 += sd.chunk) {
    const int tc = (int)std::min<int64_t>(sd.chunk, D.T - t0);
    const void* nf_c = at((const void*)K.nf, (size_t)t0 * D.d, es);
    {  // logits = nf W
      GemmDesc g;
      if (sd.tied) g = gemm1(tc, V, D.d, nf_c, D.d, 1, w->embedding, D.d, 1, ty);
      else if (head_mfma) g = gemm1(tc, V, D.d, nf_c, D.d, 1, K.wout_t, D.d, 1, ty);
      else g = gemm1(tc, V, D.d, nf_c, D.d, 1, w->logits_w, V, 0, ty);
      T5_STEP("gemm_logits", run_gemm(g, epi(EPI_STORE, K.logits, V, ty), st));
    }
    T5_STEP("xent_rows", launch_xent_rows(K.logits, ty, targets + t0, tc, V, V, cfg->z_loss, K.n_valid,
                                          K.loss_rows + t0, grads ? 1 : 0, st));
    if (!grads) continue;
    {  // dnf = dlogits W^T
      GemmDesc g;
      if (!sd.tied) g = gemm1(tc, D.d, V, K.logits, V, 1, w->logits_w, V, 1, ty);
      else if (head_mfma) g = gemm1(tc, D.d, V, K.logits, V, 1, K.wout_t, V, 1, ty);
      else g = gemm1(tc, D.d, V, K.logits, V, 1, w->embedding, D.d, 0, ty);
      T5_STEP("gemm_dnf", run_gemm(g, epi(EPI_STORE, K.dnf + (size_t)t0 * D.d, D.d, IN_F32), st));
    }
    if (sd.tied) {  // dE += dlogits^T nf'
      GemmDesc g = gemm1(V, D.d, tc, K.logits, V, 0, nf_c, D.d, 0, ty);
      GemmEpi e = epi(EPI_SPLIT_F32, grads->embedding, D.d, IN_F32);
      e.accumulate = 1;
      T5_STEP("gemm_dlogits_w", run_gemm(g, e, st));
    } else {  // dWout += nf^T dlogits
      GemmDesc g = gemm1(D.d, V, tc, nf_c, D.d, 0, K.logits, V, 0, ty);
      GemmEpi e = epi(EPI_SPLIT_F32, grads->logits_w, V, IN_F32);
      e.accumulate = 1;
      T5_STEP("gemm_dlogits_w", run_gemm(g, e, st));
    }
  }
  T5_STEP("loss_reduce", launch_loss_reduce(K.loss_rows, D.T, K.n_valid, loss, st));
  if (!grads) return T5_OK;

  // ---------------------------------------------------------------- backward sweep
  BwdWs BW;
  carve_bwd(D, K.block_ws, &BW);
  BW.ddiag = K.ddiag;
  {
    ZeroList z;
    std::memset(&z, 0, sizeof(z));
    z.p[0] = K.ddiag; z.n[0] = (int64_t)D.H * (2 * D.S - 1); z.count = 1;
    T5_STEP("zero_grads", launch_zero_f32(z, st));
  }
  // gradient of x_L through the final norm (no residual term)
  if (sd.tied) {
    T5_STEP("rmsnorm_bwd", launch_rmsnorm_bwd(x_of(sd.L), ty, gf, ty, K.rf, K.dnf, nullptr, IN_F32,
                                              ty == IN_F32 ? (float*)K.dxa : nullptr, ty == IN_BF16 ? K.dxa : nullptr,
                                              ty, K.dg_tmp, BW.dg_partial, 0, T, D.d, st));
    T5_STEP("axpy", launch_axpy_f32(grads->final_scale, K.dg_tmp, s_tied, D.d, acc, st));
  } else {
    T5_STEP("rmsnorm_bwd", launch_rmsnorm_bwd(x_of(sd.L), ty, gf, ty, K.rf, K.dnf, nullptr, IN_F32,
                                              ty == IN_F32 ? (float*)K.dxa : nullptr, ty == IN_BF16 ? K.dxa : nullptr,
                                              ty, grads->final_scale, BW.dg_partial, acc, T, D.d, st));
  }
  const AttnDims ad = self_dims(bc, D);
  const int far = lut.n_thr > 0 ? lut.thr[lut.n_thr - 1] : lut.max_exact;
  const bool attn_mfma = ty == IN_BF16 && attn_mfma_supported(ad) && attn_bwd_mfma_fits(ad, far);
  void* dy = K.dxa;
  void* dx = K.dxb;
  for (int l = sd.L - 1; l >= 0; --l) {
    if (sd.remat) T5_SUB(layer_fwd(l));  // rebuilds layer l's saved activations (and x_{l+1}, unchanged)
    Stash S;
    carve_stash(D, stash_of(l), &S);
    S.diag = K.diag;
    T5_SUB(bwd_zero(D, &lg[l], nullptr, nullptr, acc != 0, st));
    T5_SUB(bwd_mlp(D, dy, S.h, &lw[l], S, BW, &lg[l], acc, st));
    T5_SUB(bwd_self_attn(bc, D, lut, x_of(l), BW.dh, BW.dh_lp, &lw[l], S, BW, attn_mfma, far, dx, &lg[l], acc, st,
                         false));
    std::swap(dy, dx);
  }
  // dy now holds the gradient of x_0
  T5_STEP("relpos_diag_bwd", launch_relpos_diag_bwd(K.ddiag, grads->rel_table, D.S, D.H, bc->num_buckets, lut, acc, st));
  T5_STEP("embed_bwd", launch_embed_bwd(tokens, dy, ty, grads->embedding, D.T, D.d, V, st));
  return T5_OK;
}

}  // extern "C"
