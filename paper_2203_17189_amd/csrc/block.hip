// C-ABI entry points of the T5.1.1 block, the decoder layer and Adafactor (see include/t5mi.h).
// All validation happens before the first HIP call.
#include "block_host.h"

namespace t5mi {
bool g_timing = false;
std::vector<StepRec> g_recs;
SideStream g_side;
}  // namespace t5mi

namespace {
constexpr int kAfMaxListed = 1 << 16;  // tensors one adafactor_step_multi call may list
}

extern "C" {

const char* t5_status_string(int s) {
  switch (s) {
    case T5_OK: return "ok";
    case T5_ERR_NULL: return "null pointer";
    case T5_ERR_SHAPE: return "invalid shape or hyper-parameter";
    case T5_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case T5_ERR_WORKSPACE: return "workspace too small";
    case T5_ERR_DEVICE: return "HIP launch failed";
    default: return "unknown status";
  }
}

int t5_relpos_bucket(const int32_t* rel_pos, int32_t* bucket, int64_t n, int bidirectional, int num_buckets,
                     int max_distance, void* stream) {
  if (n < 0) return T5_ERR_SHAPE;
  RelposLut lut;
  const int rc = relpos_build_lut(bidirectional, num_buckets, max_distance, &lut);
  if (rc != T5_OK) return rc;
  if (n == 0) return T5_OK;
  if (!rel_pos || !bucket) return T5_ERR_NULL;
  T5_TRY(launch_relpos_bucket(rel_pos, bucket, n, lut, (hipStream_t)stream));
  return T5_OK;
}

int t5_dropout_keep(uint64_t seed, int site, float rate, int64_t rows, int64_t cols, uint8_t* keep, void* stream) {
  if (rows < 0 || cols < 0 || !(rate >= 0.f && rate < 1.f)) return T5_ERR_SHAPE;
  if (rows > ((int64_t)1 << 32) || cols > ((int64_t)1 << 32)) return T5_ERR_UNSUPPORTED;
  if (rows == 0 || cols == 0) return T5_OK;
  if (!keep) return T5_ERR_NULL;
  hipStream_t st = (hipStream_t)stream;
  T5_STEP("dropout_keep", launch_dropout_keep(make_drop_site(seed, site, rate), rows, cols, keep, st));
  return T5_OK;
}

size_t t5_block_stash_bytes(const t5_block_cfg* cfg) {
  Dims D;
  if (validate_cfg(cfg, &D, nullptr) != T5_OK) return 0;
  return carve_stash(D, nullptr, nullptr);
}

size_t t5_block_workspace_bytes(const t5_block_cfg* cfg) {
  Dims D;
  if (validate_cfg(cfg, &D, nullptr) != T5_OK) return 0;
  const size_t f = carve_fwd(D, nullptr, nullptr), b = carve_bwd(D, nullptr, nullptr);
  return f > b ? f : b;
}

size_t t5_decoder_block_stash_bytes(const t5_block_cfg* cfg, int32_t enc_seq) {
  Dims D;
  if (enc_seq < 1 || validate_cfg(cfg, &D, nullptr, enc_seq) != T5_OK) return 0;
  return carve_stash(D, nullptr, nullptr);
}

size_t t5_decoder_block_workspace_bytes(const t5_block_cfg* cfg, int32_t enc_seq) {
  Dims D;
  if (enc_seq < 1 || validate_cfg(cfg, &D, nullptr, enc_seq) != T5_OK) return 0;
  const size_t f = carve_fwd(D, nullptr, nullptr), b = carve_bwd(D, nullptr, nullptr);
  return f > b ? f : b;
}

int t5_block_kernel_path(const t5_block_cfg* cfg, int32_t enc_seq) {
  Dims D;
  RelposLut lut;
  if (enc_seq < 0 || validate_cfg(cfg, &D, &lut, enc_seq) != T5_OK) return -1;
  int path = 0;
  if (fused_fwd_ok(D)) path |= T5_PATH_MFMA_GEMM;
  const AttnDims ad = self_dims(cfg, D);
  const int far = lut.n_thr > 0 ? lut.thr[lut.n_thr - 1] : lut.max_exact;
  if (D.ty == IN_BF16 && attn_mfma_supported(ad)) {
    path |= T5_PATH_MFMA_ATTN_FWD;
    if (attn_bwd_mfma_fits(ad, far)) path |= T5_PATH_MFMA_ATTN_BWD;
  }
  if (enc_seq > 0 && D.ty == IN_BF16 && attn_mfma_supported(cross_dims(cfg, D))) path |= T5_PATH_MFMA_CROSS_ATTN;
  return path;
}

int t5_block_fwd(const t5_block_cfg* cfg, const void* x, const t5_block_weights* w, void* y, void* stash,
                 void* workspace, size_t workspace_bytes, void* stream) {
  Dims D;
  RelposLut lut;
  const int rc = validate_cfg(cfg, &D, &lut);
  if (rc != T5_OK) return rc;
  if (!x || !w || !y || !stash || !workspace) return T5_ERR_NULL;
  if (!weights_present(w, D)) return T5_ERR_NULL;
  if (workspace_bytes < carve_fwd(D, nullptr, nullptr)) return T5_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  Stash S;
  carve_stash(D, stash, &S);
  FwdWs W;
  carve_fwd(D, workspace, &W);
  const bool fused = fused_fwd_ok(D);
  if (fused) T5_SUB(fwd_pack_weights(D, w, nullptr, W, st));
  T5_SUB(fwd_self_attn(cfg, D, lut, x, w, S, W, fused, st));
  T5_SUB(fwd_mlp(cfg, D, S.h, w, S, W, fused, y, st));
  return T5_OK;
}

int t5_block_bwd(const t5_block_cfg* cfg, const void* dy, const void* x, const t5_block_weights* w,
                 const void* stash, void* dx, const t5_block_grads* dw, int accumulate, void* workspace,
                 size_t workspace_bytes, void* stream) {
  Dims D;
  RelposLut lut;
  const int rc = validate_cfg(cfg, &D, &lut);
  if (rc != T5_OK) return rc;
  if (!dy || !x || !w || !stash || !dx || !dw || !workspace) return T5_ERR_NULL;
  if (!weights_present(w, D) || !grads_present(dw, D)) return T5_ERR_NULL;
  if (workspace_bytes < carve_bwd(D, nullptr, nullptr)) return T5_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  Stash S;
  carve_stash(D, const_cast<void*>(stash), &S);
  BwdWs W;
  carve_bwd(D, workspace, &W);
  const int acc = accumulate ? 1 : 0;
  const AttnDims ad = self_dims(cfg, D);
  const int far = lut.n_thr > 0 ? lut.thr[lut.n_thr - 1] : lut.max_exact;
  const bool attn_mfma = D.ty == IN_BF16 && attn_mfma_supported(ad) && attn_bwd_mfma_fits(ad, far);
  W.fork = fork_begin(st, D.drop == 0.f && !D.det);
  ForkGuard guard(W.fork);
  T5_SUB(bwd_zero(D, dw, nullptr, attn_mfma ? W.ddiag : nullptr, acc != 0, st));
  T5_SUB(bwd_mlp(D, dy, S.h, w, S, W, dw, acc, st));
  T5_SUB(bwd_self_attn(cfg, D, lut, x, W.dh, W.dh_lp, w, S, W, attn_mfma, far, dx, dw, acc, st));
  T5_TRY(guard.join());
  return T5_OK;
}

int t5_decoder_block_fwd(const t5_block_cfg* cfg, int32_t enc_seq, const void* x, const void* enc,
                         const t5_block_weights* w, const t5_cross_weights* xw, void* y, void* stash,
                         void* workspace, size_t workspace_bytes, void* stream) {
  if (enc_seq < 1) return cfg ? T5_ERR_SHAPE : T5_ERR_NULL;
  Dims D;
  RelposLut lut;
  const int rc = validate_cfg(cfg, &D, &lut, enc_seq);
  if (rc != T5_OK) return rc;
  if (!x || !enc || !w || !xw || !y || !stash || !workspace) return T5_ERR_NULL;
  if (!weights_present(w, D)) return T5_ERR_NULL;
  if (!xw->lnx_scale || !xw->xq || !xw->xk || !xw->xv || !xw->xo) return T5_ERR_NULL;
  if (workspace_bytes < carve_fwd(D, nullptr, nullptr)) return T5_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  Stash S;
  carve_stash(D, stash, &S);
  FwdWs W;
  carve_fwd(D, workspace, &W);
  const bool fused = fused_fwd_ok(D);
  if (fused) T5_SUB(fwd_pack_weights(D, w, xw, W, st));
  T5_SUB(fwd_self_attn(cfg, D, lut, x, w, S, W, fused, st));
  T5_SUB(fwd_cross_attn(cfg, D, enc, xw, S, W, fused, st));
  T5_SUB(fwd_mlp(cfg, D, S.h2, w, S, W, fused, y, st));
  return T5_OK;
}

int t5_decoder_block_bwd(const t5_block_cfg* cfg, int32_t enc_seq, const void* dy, const void* x,
                         const void* enc, const t5_block_weights* w, const t5_cross_weights* xw,
                         const void* stash, void* dx, void* denc, const t5_block_grads* dw,
                         const t5_cross_grads* dxw, int accumulate, void* workspace, size_t workspace_bytes,
                         void* stream) {
  if (enc_seq < 1) return cfg ? T5_ERR_SHAPE : T5_ERR_NULL;
  Dims D;
  RelposLut lut;
  const int rc = validate_cfg(cfg, &D, &lut, enc_seq);
  if (rc != T5_OK) return rc;
  if (!dy || !x || !enc || !w || !xw || !stash || !dx || !denc || !dw || !dxw || !workspace) return T5_ERR_NULL;
  if (!weights_present(w, D) || !grads_present(dw, D)) return T5_ERR_NULL;
  if (!xw->lnx_scale || !xw->xq || !xw->xk || !xw->xv || !xw->xo) return T5_ERR_NULL;
  if (!dxw->lnx_scale || !dxw->xq || !dxw->xk || !dxw->xv || !dxw->xo) return T5_ERR_NULL;
  if (workspace_bytes < carve_bwd(D, nullptr, nullptr)) return T5_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  Stash S;
  carve_stash(D, const_cast<void*>(stash), &S);
  BwdWs W;
  carve_bwd(D, workspace, &W);
  const int acc = accumulate ? 1 : 0;
  const AttnDims ad = self_dims(cfg, D);
  const int far = lut.n_thr > 0 ? lut.thr[lut.n_thr - 1] : lut.max_exact;
  const bool attn_mfma = D.ty == IN_BF16 && attn_mfma_supported(ad) && attn_bwd_mfma_fits(ad, far);
  W.fork = fork_begin(st, D.drop == 0.f && !D.det);
  ForkGuard guard(W.fork);
  T5_SUB(bwd_zero(D, dw, dxw, attn_mfma ? W.ddiag : nullptr, acc != 0, st));
  T5_SUB(bwd_mlp(D, dy, S.h2, w, S, W, dw, acc, st));
  T5_SUB(bwd_cross_attn(cfg, D, enc, xw, S, W, denc, dxw, acc, st));
  T5_SUB(bwd_self_attn(cfg, D, lut, x, W.dh1, W.dh1_lp, w, S, W, attn_mfma, far, dx, dw, acc, st));
  T5_TRY(guard.join());
  return T5_OK;
}

int t5_gemm_bf16(const void* A, const void* B, float* C, int M, int N, int K, int lda, int ldb, int ldc, int a_kc,
                 int b_kc, void* stream) {
  if (M < 1 || N < 1 || K < 1 || lda < 1 || ldb < 1 || ldc < N) return T5_ERR_SHAPE;
  if (!A || !B || !C) return T5_ERR_NULL;
  GemmDesc g = gemm1(M, N, K, A, lda, a_kc ? 1 : 0, B, ldb, b_kc ? 1 : 0, IN_BF16);
  GemmEpi e = a_kc ? epi(EPI_STORE, C, ldc, IN_F32) : epi(EPI_SPLIT_F32, C, ldc, IN_F32);
  if (!gemm_mfma_supported(g, e)) return T5_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  T5_STEP("gemm_bf16", launch_gemm_mfma(g, e, st));
  return T5_OK;
}

int t5_wgrad_overlap_enable(int enable) {
  if (!enable) {
    if (g_side.stream) {
      (void)hipStreamSynchronize(g_side.stream);
      (void)hipEventDestroy(g_side.ev_fork);
      (void)hipEventDestroy(g_side.ev_join);
      (void)hipStreamDestroy(g_side.stream);
      g_side = SideStream();
    }
    return T5_OK;
  }
  if (g_side.stream) return T5_OK;
  SideStream s;
  if (hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking) != hipSuccess) return T5_ERR_DEVICE;  // default priority
  if (hipEventCreateWithFlags(&s.ev_fork, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&s.ev_join, hipEventDisableTiming) != hipSuccess) {
    (void)hipStreamDestroy(s.stream);
    return T5_ERR_DEVICE;
  }
  g_side = s;
  return T5_OK;
}

void t5_step_timing_enable(int enable) {
  for (auto& r : g_recs) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
  g_recs.clear();
  g_timing = enable != 0;
}

int t5_step_timing_read(const char** names, float* ms, int* calls, int cap) {
  int n = 0;
  for (auto& r : g_recs) {
    if (hipEventSynchronize(r.e1) != hipSuccess) continue;
    float t = 0.f;
    if (hipEventElapsedTime(&t, r.e0, r.e1) != hipSuccess) continue;
    int k = 0;
    while (k < n && std::strcmp(names[k], r.name) != 0) ++k;
    if (k == n) {
      if (n >= cap) continue;
      names[n] = r.name; ms[n] = 0.f; calls[n] = 0; ++n;
    }
    ms[k] += t;
    calls[k] += 1;
  }
  return n;
}

size_t adafactor_workspace_bytes(int64_t rows, int64_t cols, int factored) {
  if (rows < 1 || cols < 1) return 0;
  return adafactor_ws_bytes(rows, cols, factored);
}

int adafactor_step(float* param, const float* grad, float* v_row, float* v_col, float* v_full, int64_t rows,
                   int64_t cols, int factored, const adafactor_cfg* cfg, void* bf16_copy_out, void* workspace,
                   size_t workspace_bytes, void* stream) {
  if (!cfg) return T5_ERR_NULL;
  if (rows < 1 || cols < 1 || cfg->step < 1 || !(cfg->clip > 0.f) || !(cfg->eps1 >= 0.f)) return T5_ERR_SHAPE;
  if (!(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->weight_decay >= 0.f)) return T5_ERR_SHAPE;
  if (cfg->beta1 > 0.f) return T5_ERR_UNSUPPORTED;
  if (rows > (1 << 24) || cols > (1 << 24)) return T5_ERR_UNSUPPORTED;
  if (!param || !grad || !workspace) return T5_ERR_NULL;
  if (factored ? (!v_row || !v_col) : !v_full) return T5_ERR_NULL;
  if (workspace_bytes < adafactor_ws_bytes(rows, cols, factored)) return T5_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  T5_STEP("adafactor", launch_adafactor(param, grad, v_row, v_col, v_full, rows, cols, factored, *cfg, bf16_copy_out,
                                        workspace, st));
  return T5_OK;
}

// Tensors are processed in groups of AF_MAX_TENSORS consecutive entries (one launch sequence each, in
// stream order), so the groups share one workspace: the largest group's.
size_t adafactor_multi_workspace_bytes(const adafactor_tensor* t, int n) {
  if (!t || n < 1 || n > kAfMaxListed) return 0;
  size_t need = 0;
  for (int i0 = 0; i0 < n; i0 += AF_MAX_TENSORS) {
    size_t total = 0;
    for (int i = i0; i < n && i < i0 + AF_MAX_TENSORS; ++i) {
      if (t[i].rows < 1 || t[i].cols < 1) return 0;
      total += adafactor_ws_bytes(t[i].rows, t[i].cols, t[i].factored);
    }
    need = total > need ? total : need;
  }
  return need;
}

int adafactor_step_multi(const adafactor_tensor* t, int n, const adafactor_cfg* cfg, void* workspace,
                         size_t workspace_bytes, void* stream) {
  if (!cfg || !t) return T5_ERR_NULL;
  if (n < 1) return T5_ERR_SHAPE;
  if (n > kAfMaxListed) return T5_ERR_UNSUPPORTED;
  if (cfg->step < 1 || !(cfg->clip > 0.f) || !(cfg->eps1 >= 0.f)) return T5_ERR_SHAPE;
  if (!(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->weight_decay >= 0.f)) return T5_ERR_SHAPE;
  for (int i = 0; i < n; ++i) {  // every entry is checked before the first launch
    if (t[i].rows < 1 || t[i].cols < 1) return T5_ERR_SHAPE;
    if (t[i].rows > (1 << 24) || t[i].cols > (1 << 24)) return T5_ERR_UNSUPPORTED;
    if (!t[i].param || !t[i].grad) return T5_ERR_NULL;
    if (t[i].factored ? (!t[i].v_row || !t[i].v_col) : !t[i].v_full) return T5_ERR_NULL;
    if (cfg->beta1 > 0.f && !t[i].m) return T5_ERR_NULL;
  }
  if (!workspace) return T5_ERR_NULL;
  if (workspace_bytes < adafactor_multi_workspace_bytes(t, n)) return T5_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  for (int i0 = 0; i0 < n; i0 += AF_MAX_TENSORS) {
    AfTensor items[AF_MAX_TENSORS];
    const int m = n - i0 < AF_MAX_TENSORS ? n - i0 : AF_MAX_TENSORS;
    for (int i = 0; i < m; ++i) {
      const adafactor_tensor& a = t[i0 + i];
      items[i] = AfTensor{a.param, a.grad, a.v_row, a.v_col, a.v_full, a.rows, a.cols, a.factored, a.bf16_copy_out, a.m};
    }
    T5_STEP("adafactor", launch_adafactor_multi(items, m, *cfg, workspace, st));
  }
  return T5_OK;
}

int t5_mfma_peak_probe(int workgroups, int iters, int random_operands, float* sink, void* stream) {
  if (workgroups < 1 || iters < 1 || workgroups > (1 << 20)) return T5_ERR_SHAPE;
  if (!sink) return T5_ERR_NULL;
  hipStream_t st = (hipStream_t)stream;
  T5_STEP("mfma_peak_probe", launch_mfma_peak_probe(workgroups, iters, random_operands, sink, st));
  return T5_OK;
}

}  // extern "C"
