// C-ABI entry points and host-side sequencing of the T5.1.1 block (see include/t5mi.h).
// All validation happens before the first HIP call.
#include <cmath>
#include <cstring>
#include <string>
#include <vector>
#include "kernels.h"

using namespace t5mi;

namespace {

struct Dims {
  int B, S, d, H, dk, F, I;
  int64_t T;
  size_t es;  // bytes per stored element
  int ty;     // IN_F32 / IN_BF16
};

int validate_cfg(const t5_block_cfg* c, Dims* o, RelposLut* lut) {
  if (!c) return T5_ERR_NULL;
  if (c->batch < 1 || c->seq < 1 || c->d_model < 1 || c->n_heads < 1 || c->d_kv < 1 || c->d_ff < 1)
    return T5_ERR_SHAPE;
  if (c->dtype != T5_F32 && c->dtype != T5_BF16) return T5_ERR_UNSUPPORTED;
  if (!(c->rms_eps >= 0.f) || !std::isfinite(c->attn_scale)) return T5_ERR_SHAPE;
  const int64_t T = (int64_t)c->batch * c->seq;
  const int64_t I = (int64_t)c->n_heads * c->d_kv;
  if (T > (1 << 24) || I > (1 << 16) || c->d_model > (1 << 16) || c->d_ff > (1 << 18) || c->seq > (1 << 16))
    return T5_ERR_UNSUPPORTED;
  if (c->d_model > 8192 || (c->d_model % 8 != 0 && c->d_model > 1024)) return T5_ERR_UNSUPPORTED;
  RelposLut tmp;
  const int rc = relpos_build_lut(c->causal ? 0 : 1, c->num_buckets, c->max_distance, lut ? lut : &tmp);
  if (rc != T5_OK) return rc;
  if (o) {
    o->B = c->batch; o->S = c->seq; o->d = c->d_model; o->H = c->n_heads; o->dk = c->d_kv; o->F = c->d_ff;
    o->I = (int)I; o->T = T;
    o->ty = c->dtype == T5_BF16 ? IN_BF16 : IN_F32;
    o->es = c->dtype == T5_BF16 ? 2 : 4;
  }
  return T5_OK;
}

// Bump allocator over a caller-provided buffer; with base == nullptr it only measures.
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base((char*)b) {}
  template <typename T = void>
  T* take(size_t bytes) {
    char* p = base ? base + off : nullptr;
    off += align_up(bytes);
    return (T*)p;
  }
};

struct Stash {
  float *r1, *r2, *lse, *h, *diag;
  // gp = w * gelu'(u) and gl = gelu(u) are the saved factors of the gated GELU (u, w: the wi_0 / wi_1
  // projections); the simple path uses the two buffers for u and w first and converts them in place.
  void *n1, *qkv, *c, *n2, *gp, *gl, *a;
};
size_t carve_stash(const Dims& D, void* base, Stash* s) {
  Carver cv(base);
  Stash t;
  t.r1 = cv.take<float>(D.T * 4);
  t.r2 = cv.take<float>(D.T * 4);
  t.lse = cv.take<float>((size_t)D.B * D.H * D.S * 4);
  t.diag = cv.take<float>((size_t)D.H * (2 * D.S - 1) * 4);
  t.h = cv.take<float>((size_t)D.T * D.d * 4);
  t.n1 = cv.take((size_t)D.T * D.d * D.es);
  t.qkv = cv.take((size_t)D.T * 3 * D.I * D.es);
  t.c = cv.take((size_t)D.T * D.I * D.es);
  t.n2 = cv.take((size_t)D.T * D.d * D.es);
  t.gp = cv.take((size_t)D.T * D.F * D.es);
  t.gl = cv.take((size_t)D.T * D.F * D.es);
  t.a = cv.take((size_t)D.T * D.F * D.es);
  if (s) *s = t;
  return cv.off;
}

struct FwdWs {
  void *wqkv_t, *wo_t, *wi_t, *woff_t;  // packed transposed weights (bf16 MFMA path)
};
size_t carve_fwd(const Dims& D, void* base, FwdWs* w) {
  Carver cv(base);
  FwdWs t;
  t.wqkv_t = cv.take((size_t)3 * D.I * D.d * D.es);
  t.wo_t = cv.take((size_t)D.d * D.I * D.es);
  t.wi_t = cv.take((size_t)2 * D.F * D.d * D.es);
  t.woff_t = cv.take((size_t)D.d * D.F * D.es);
  if (w) *w = t;
  return cv.off;
}

struct BwdWs {
  float *dn, *dh, *dvec, *ddiag, *dg_partial;
  void *dh_lp, *duw, *dc, *dqkv, *attn_scratch;  // duw: [T][2F], du in columns 0..F-1, dw in F..2F-1
};
size_t carve_bwd(const Dims& D, void* base, BwdWs* w) {
  Carver cv(base);
  BwdWs t;
  t.dn = cv.take<float>((size_t)D.T * D.d * 4);
  t.dh = cv.take<float>((size_t)D.T * D.d * 4);
  t.dvec = cv.take<float>((size_t)D.B * D.H * D.S * 4);
  t.ddiag = cv.take<float>((size_t)D.H * (2 * D.S - 1) * 4);
  t.dg_partial = cv.take<float>((size_t)rmsnorm_bwd_partial_rows((int)D.T) * D.d * 4);
  t.dh_lp = cv.take(D.ty == IN_BF16 ? (size_t)D.T * D.d * D.es : 0);
  t.duw = cv.take((size_t)D.T * 2 * D.F * D.es);
  t.dc = cv.take((size_t)D.T * D.I * D.es);
  t.dqkv = cv.take((size_t)D.T * 3 * D.I * D.es);
  AttnDims ad{D.B, D.S, D.H, D.dk, 0, 1.f};
  t.attn_scratch = cv.take(attn_bwd_mfma_scratch_bytes(ad));
  if (w) *w = t;
  return cv.off;
}

inline const void* at(const void* p, size_t elems, size_t es) { return (const char*)p + elems * es; }
inline void* at(void* p, size_t elems, size_t es) { return (char*)p + elems * es; }

GemmDesc gemm1(int M, int N, int K, const void* A, int lda, int a_kc, const void* B, int ldb, int b_kc,
               int ty) {
  GemmDesc g;
  std::memset(&g, 0, sizeof(g));
  g.M = M; g.N = N; g.nseg = 1;
  g.seg[0] = GemmSeg{A, B, lda, ldb, K};
  g.a_kc = a_kc; g.b_kc = b_kc; g.in_type = ty;
  return g;
}
GemmEpi epi(int kind, void* out0, int ld0, int out_type) {
  GemmEpi e;
  std::memset(&e, 0, sizeof(e));
  e.kind = kind; e.out0 = out0; e.ld0 = ld0; e.out_type = out_type; e.split_n = 1 << 30;
  return e;
}

hipError_t run_gemm(const GemmDesc& g, const GemmEpi& e, hipStream_t st) {
  if (gemm_mfma_supported(g, e)) return launch_gemm_mfma(g, e, st);
  return launch_gemm_simple(g, e, st);
}

#define T5_TRY(expr)                          \
  do {                                        \
    if ((expr) != hipSuccess) return T5_ERR_DEVICE; \
  } while (0)

// ---- optional per-step device timing (see t5_step_timing_enable in the header)
struct StepRec {
  const char* name;
  hipEvent_t e0, e1;
};
bool g_timing = false;
std::vector<StepRec> g_recs;

struct StepScope {
  hipStream_t st;
  bool on;
  StepRec rec;
  StepScope(const char* name, hipStream_t s) : st(s), on(g_timing) {
    if (!on) return;
    rec.name = name;
    if (hipEventCreate(&rec.e0) != hipSuccess || hipEventCreate(&rec.e1) != hipSuccess) { on = false; return; }
    (void)hipEventRecord(rec.e0, st);
  }
  ~StepScope() {
    if (!on) return;
    (void)hipEventRecord(rec.e1, st);
    g_recs.push_back(rec);
  }
};
#define T5_STEP(name, expr)                           \
  do {                                                \
    StepScope scope_(name, st);                       \
    if ((expr) != hipSuccess) return T5_ERR_DEVICE;   \
  } while (0)

bool fused_fwd_ok(const Dims& D) {
  // The packed-weight MFMA forward needs the MFMA GEMM for every projection of this shape; the
  // fused gated-GELU GEMM is the most demanding one, so probe it with placeholder pointers.
  if (D.ty != IN_BF16 || D.d % 64 != 0 || D.I % 64 != 0 || D.F % 64 != 0) return false;
  static const long long dummy[4] = {0, 0, 0, 0};
  GemmDesc g = gemm1((int)D.T, 2 * D.F, D.d, dummy, D.d, 1, dummy, D.d, 1, IN_BF16);
  GemmEpi e = epi(EPI_GEGLU_FWD, (void*)dummy, D.F, IN_BF16);
  e.out1 = (void*)dummy; e.out2 = (void*)dummy;
  return gemm_mfma_supported(g, e);
}

}  // namespace

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

int t5_block_fwd(const t5_block_cfg* cfg, const void* x, const t5_block_weights* w, void* y, void* stash,
                 void* workspace, size_t workspace_bytes, void* stream) {
  Dims D;
  RelposLut lut;
  const int rc = validate_cfg(cfg, &D, &lut);
  if (rc != T5_OK) return rc;
  if (!x || !w || !y || !stash || !workspace) return T5_ERR_NULL;
  if (!w->ln1_scale || !w->wq || !w->wk || !w->wv || !w->wo || !w->rel_table || !w->ln2_scale || !w->wi0 ||
      !w->wi1 || !w->wo_ff)
    return T5_ERR_NULL;
  if (workspace_bytes < carve_fwd(D, nullptr, nullptr)) return T5_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  Stash S;
  carve_stash(D, stash, &S);
  FwdWs W;
  carve_fwd(D, workspace, &W);
  const int T = (int)D.T, ty = D.ty;
  const size_t es = D.es;
  const AttnDims ad{D.B, D.S, D.H, D.dk, cfg->causal ? 1 : 0, cfg->attn_scale};
  const bool fused = fused_fwd_ok(D);

  T5_STEP("relpos_diag", launch_relpos_diag(w->rel_table, cfg->dtype, S.diag, D.S, D.H, lut, st));
  T5_STEP("rmsnorm_fwd", launch_rmsnorm_fwd(x, ty, w->ln1_scale, S.n1, ty, S.r1, T, D.d, cfg->rms_eps, st));
  if (fused) {
    // all four weight packs (transposes to k-contiguous rows) in one launch
    PackJobs pj;
    std::memset(&pj, 0, sizeof(pj));
    pj.j[0] = PackJob{{w->wq, w->wk, w->wv}, 3, D.d, D.I, 0, W.wqkv_t};
    pj.j[1] = PackJob{{w->wo, nullptr, nullptr}, 1, D.I, D.d, 0, W.wo_t};
    pj.j[2] = PackJob{{w->wi0, w->wi1, nullptr}, 2, D.d, D.F, 32, W.wi_t};
    pj.j[3] = PackJob{{w->wo_ff, nullptr, nullptr}, 1, D.F, D.d, 0, W.woff_t};
    pj.count = 4;
    T5_STEP("pack_weights", launch_pack_transpose_multi(pj, st));
    GemmDesc g = gemm1(T, 3 * D.I, D.d, S.n1, D.d, 1, W.wqkv_t, D.d, 1, ty);
    T5_STEP("gemm_qkv", run_gemm(g, epi(EPI_STORE, S.qkv, 3 * D.I, ty), st));
  } else {
    const void* ws3[3] = {w->wq, w->wk, w->wv};
    for (int j = 0; j < 3; ++j) {
      GemmDesc g = gemm1(T, D.I, D.d, S.n1, D.d, 1, ws3[j], D.I, 0, ty);
      T5_STEP("gemm_qkv", run_gemm(g, epi(EPI_STORE, at(S.qkv, (size_t)j * D.I, es), 3 * D.I, ty), st));
    }
  }
  if (ty == IN_BF16 && attn_mfma_supported(ad))
    T5_STEP("attn_fwd", launch_attn_fwd_mfma(S.qkv, S.diag, S.c, S.lse, ad, st));
  else
    T5_STEP("attn_fwd", launch_attn_fwd_simple(S.qkv, ty, S.diag, S.c, S.lse, ad, st));
  {  // h = x + c Wo  (float32 residual stream)
    GemmDesc g;
    if (fused) {
      g = gemm1(T, D.d, D.I, S.c, D.I, 1, W.wo_t, D.I, 1, ty);
    } else {
      g = gemm1(T, D.d, D.I, S.c, D.I, 1, w->wo, D.d, 0, ty);
    }
    GemmEpi e = epi(EPI_RESID, S.h, D.d, IN_F32);
    e.aux0 = x; e.aux_type = ty;
    T5_STEP("gemm_o", run_gemm(g, e, st));
  }
  T5_STEP("rmsnorm_fwd", launch_rmsnorm_fwd(S.h, IN_F32, w->ln2_scale, S.n2, ty, S.r2, T, D.d, cfg->rms_eps, st));
  if (fused) {
    GemmDesc g = gemm1(T, 2 * D.F, D.d, S.n2, D.d, 1, W.wi_t, D.d, 1, ty);
    GemmEpi e = epi(EPI_GEGLU_FWD, S.gp, D.F, ty);
    e.out1 = S.gl; e.out2 = S.a;
    if (!gemm_mfma_supported(g, e)) return T5_ERR_UNSUPPORTED;
    T5_STEP("gemm_wi_geglu", launch_gemm_mfma(g, e, st));
  } else {
    GemmDesc g0 = gemm1(T, D.F, D.d, S.n2, D.d, 1, w->wi0, D.F, 0, ty);
    T5_STEP("gemm_wi", run_gemm(g0, epi(EPI_STORE, S.gp, D.F, ty), st));
    GemmDesc g1 = gemm1(T, D.F, D.d, S.n2, D.d, 1, w->wi1, D.F, 0, ty);
    T5_STEP("gemm_wi", run_gemm(g1, epi(EPI_STORE, S.gl, D.F, ty), st));
    T5_STEP("geglu_fwd", launch_geglu_fwd(S.gp, S.gl, S.a, ty, (int64_t)D.T * D.F, st));
  }
  {  // y = h + a Wo_ff
    GemmDesc g;
    if (fused) {
      g = gemm1(T, D.d, D.F, S.a, D.F, 1, W.woff_t, D.F, 1, ty);
    } else {
      g = gemm1(T, D.d, D.F, S.a, D.F, 1, w->wo_ff, D.d, 0, ty);
    }
    GemmEpi e = epi(EPI_RESID, y, D.d, ty);
    e.aux0 = S.h; e.aux_type = IN_F32;
    T5_STEP("gemm_wo", run_gemm(g, e, st));
  }
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
  if (!w->ln1_scale || !w->wq || !w->wk || !w->wv || !w->wo || !w->rel_table || !w->ln2_scale || !w->wi0 ||
      !w->wi1 || !w->wo_ff)
    return T5_ERR_NULL;
  if (!dw->ln1_scale || !dw->wq || !dw->wk || !dw->wv || !dw->wo || !dw->rel_table || !dw->ln2_scale ||
      !dw->wi0 || !dw->wi1 || !dw->wo_ff)
    return T5_ERR_NULL;
  if (workspace_bytes < carve_bwd(D, nullptr, nullptr)) return T5_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  Stash S;
  carve_stash(D, const_cast<void*>(stash), &S);
  BwdWs W;
  carve_bwd(D, workspace, &W);
  const int T = (int)D.T, ty = D.ty, acc = accumulate ? 1 : 0;
  const size_t es = D.es;
  const AttnDims ad{D.B, D.S, D.H, D.dk, cfg->causal ? 1 : 0, cfg->attn_scale};

  const int far = lut.n_thr > 0 ? lut.thr[lut.n_thr - 1] : lut.max_exact;
  const bool attn_mfma = ty == IN_BF16 && attn_mfma_supported(ad) && attn_bwd_mfma_fits(ad, far);
  {
    // One launch clears what later kernels add into: the weight gradients (split-k partial sums;
    // kept when the caller accumulates) and the bias-gradient diagonals of the fused attention.
    ZeroList z;
    std::memset(&z, 0, sizeof(z));
    if (attn_mfma) {
      z.p[z.count] = W.ddiag; z.n[z.count] = (int64_t)D.H * (2 * D.S - 1); ++z.count;
    }
    if (!acc) {
      float* ps[7] = {(float*)dw->wq, (float*)dw->wk, (float*)dw->wv, (float*)dw->wo, (float*)dw->wi0,
                      (float*)dw->wi1, (float*)dw->wo_ff};
      const int64_t ns[7] = {(int64_t)D.d * D.I, (int64_t)D.d * D.I, (int64_t)D.d * D.I, (int64_t)D.I * D.d,
                             (int64_t)D.d * D.F, (int64_t)D.d * D.F, (int64_t)D.F * D.d};
      for (int q = 0; q < 7; ++q) { z.p[z.count] = ps[q]; z.n[z.count] = ns[q]; ++z.count; }
    }
    if (z.count > 0) T5_STEP("zero_grads", launch_zero_f32(z, st));
  }
  void* du_p = W.duw;
  void* dw_p = at(W.duw, (size_t)D.F, es);
  {  // dWo_ff = a^T dy
    GemmDesc g = gemm1(D.F, D.d, T, S.a, D.F, 0, dy, D.d, 0, ty);
    GemmEpi e = epi(EPI_SPLIT_F32, dw->wo_ff, D.d, IN_F32);
    e.accumulate = 1;
    T5_STEP("gemm_dwo_ff", run_gemm(g, e, st));
  }
  {  // da = dy Wo_ff^T, fused with the gated-GELU backward: du = da w gelu'(u), dw = da gelu(u)
    GemmDesc g = gemm1(T, D.F, D.d, dy, D.d, 1, w->wo_ff, D.d, 1, ty);
    GemmEpi e = epi(EPI_GEGLU_BWD, du_p, 2 * D.F, ty);
    e.out1 = dw_p; e.aux0 = S.gp; e.aux1 = S.gl; e.aux_type = ty; e.ld_aux = D.F;
    T5_STEP("gemm_da_geglu_bwd", run_gemm(g, e, st));
  }
  {  // dWi0 | dWi1 = n2^T [du | dw]
    GemmDesc g = gemm1(D.d, 2 * D.F, T, S.n2, D.d, 0, du_p, 2 * D.F, 0, ty);
    GemmEpi e = epi(EPI_SPLIT_F32, dw->wi0, D.F, IN_F32);
    e.out1 = dw->wi1; e.split_n = D.F; e.accumulate = 1;
    T5_STEP("gemm_dwi", run_gemm(g, e, st));
  }
  {  // dn2 = du Wi0^T + dw Wi1^T
    GemmDesc g = gemm1(T, D.d, D.F, du_p, 2 * D.F, 1, w->wi0, D.F, 1, ty);
    g.nseg = 2;
    g.seg[1] = GemmSeg{dw_p, w->wi1, 2 * D.F, D.F, D.F};
    T5_STEP("gemm_dn2", run_gemm(g, epi(EPI_STORE, W.dn, D.d, IN_F32), st));
  }
  // dh = dy + RMSNormBwd(h, g2, dn2)
  T5_STEP("rmsnorm_bwd", launch_rmsnorm_bwd(S.h, IN_F32, w->ln2_scale, ty, S.r2, W.dn, dy, ty, W.dh,
                            ty == IN_BF16 ? W.dh_lp : nullptr, ty, dw->ln2_scale, W.dg_partial, acc, T, D.d,
                            st));
  const void* dh_op = ty == IN_BF16 ? (const void*)W.dh_lp : (const void*)W.dh;
  {  // dWo = c^T dh
    GemmDesc g = gemm1(D.I, D.d, T, S.c, D.I, 0, dh_op, D.d, 0, ty);
    GemmEpi e = epi(EPI_SPLIT_F32, dw->wo, D.d, IN_F32);
    e.accumulate = 1;
    T5_STEP("gemm_dwo", run_gemm(g, e, st));
  }
  {  // dc = dh Wo^T
    GemmDesc g = gemm1(T, D.I, D.d, dh_op, D.d, 1, w->wo, D.d, 1, ty);
    T5_STEP("gemm_dc", run_gemm(g, epi(EPI_STORE, W.dc, D.I, ty), st));
  }
  if (attn_mfma) {
    T5_STEP("attn_bwd_prep", launch_attn_bwd_mfma(S.qkv, S.c, W.dc, S.diag, S.lse, W.dvec, W.dqkv, W.ddiag,
                                                  W.attn_scratch, ad, far, 0, st));
    T5_STEP("attn_bwd_dq", launch_attn_bwd_mfma(S.qkv, S.c, W.dc, S.diag, S.lse, W.dvec, W.dqkv, W.ddiag,
                                                W.attn_scratch, ad, far, 1, st));
    T5_STEP("attn_bwd_dkv", launch_attn_bwd_mfma(S.qkv, S.c, W.dc, S.diag, S.lse, W.dvec, W.dqkv, W.ddiag,
                                                 W.attn_scratch, ad, far, 2, st));
  }
  else
    T5_STEP("attn_bwd", launch_attn_bwd_simple(S.qkv, S.c, W.dc, ty, S.diag, S.lse, W.dvec, W.dqkv, W.ddiag, ad, st));
  T5_STEP("relpos_diag_bwd", launch_relpos_diag_bwd(W.ddiag, dw->rel_table, D.S, D.H, cfg->num_buckets, lut, acc, st));
  {  // dWq | dWk | dWv = n1^T dqkv
    GemmDesc g = gemm1(D.d, 3 * D.I, T, S.n1, D.d, 0, W.dqkv, 3 * D.I, 0, ty);
    GemmEpi e = epi(EPI_SPLIT_F32, dw->wq, D.I, IN_F32);
    e.out1 = dw->wk; e.out2 = dw->wv; e.split_n = D.I; e.accumulate = 1;
    T5_STEP("gemm_dwqkv", run_gemm(g, e, st));
  }
  {  // dn1 = dq Wq^T + dk Wk^T + dv Wv^T
    GemmDesc g = gemm1(T, D.d, D.I, W.dqkv, 3 * D.I, 1, w->wq, D.I, 1, ty);
    g.nseg = 3;
    g.seg[1] = GemmSeg{at(W.dqkv, (size_t)D.I, es), w->wk, 3 * D.I, D.I, D.I};
    g.seg[2] = GemmSeg{at(W.dqkv, (size_t)2 * D.I, es), w->wv, 3 * D.I, D.I, D.I};
    T5_STEP("gemm_dn1", run_gemm(g, epi(EPI_STORE, W.dn, D.d, IN_F32), st));
  }
  // dx = dh + RMSNormBwd(x, g1, dn1)
  T5_STEP("rmsnorm_bwd", launch_rmsnorm_bwd(x, ty, w->ln1_scale, ty, S.r1, W.dn, W.dh, IN_F32, ty == IN_F32 ? (float*)dx : nullptr,
                            ty == IN_BF16 ? dx : nullptr, ty, dw->ln1_scale, W.dg_partial, acc, T, D.d, st));
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
  if (rows > (1 << 24) || cols > (1 << 24)) return T5_ERR_UNSUPPORTED;
  if (!param || !grad || !workspace) return T5_ERR_NULL;
  if (factored ? (!v_row || !v_col) : !v_full) return T5_ERR_NULL;
  if (workspace_bytes < adafactor_ws_bytes(rows, cols, factored)) return T5_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  T5_STEP("adafactor", launch_adafactor(param, grad, v_row, v_col, v_full, rows, cols, factored, *cfg, bf16_copy_out,
                                        workspace, st));
  return T5_OK;
}

size_t adafactor_multi_workspace_bytes(const adafactor_tensor* t, int n) {
  if (!t || n < 1 || n > AF_MAX_TENSORS) return 0;
  size_t total = 0;
  for (int i = 0; i < n; ++i) {
    if (t[i].rows < 1 || t[i].cols < 1) return 0;
    total += adafactor_ws_bytes(t[i].rows, t[i].cols, t[i].factored);
  }
  return total;
}

int adafactor_step_multi(const adafactor_tensor* t, int n, const adafactor_cfg* cfg, void* workspace,
                         size_t workspace_bytes, void* stream) {
  if (!cfg || !t) return T5_ERR_NULL;
  if (n < 1) return T5_ERR_SHAPE;
  if (n > AF_MAX_TENSORS) return T5_ERR_UNSUPPORTED;
  if (cfg->step < 1 || !(cfg->clip > 0.f) || !(cfg->eps1 >= 0.f)) return T5_ERR_SHAPE;
  AfTensor items[AF_MAX_TENSORS];
  size_t need = 0;
  for (int i = 0; i < n; ++i) {
    if (t[i].rows < 1 || t[i].cols < 1) return T5_ERR_SHAPE;
    if (t[i].rows > (1 << 24) || t[i].cols > (1 << 24)) return T5_ERR_UNSUPPORTED;
    if (!t[i].param || !t[i].grad) return T5_ERR_NULL;
    if (t[i].factored ? (!t[i].v_row || !t[i].v_col) : !t[i].v_full) return T5_ERR_NULL;
    need += adafactor_ws_bytes(t[i].rows, t[i].cols, t[i].factored);
    items[i] = AfTensor{t[i].param, t[i].grad, t[i].v_row, t[i].v_col, t[i].v_full, t[i].rows, t[i].cols,
                        t[i].factored, t[i].bf16_copy_out};
  }
  if (!workspace) return T5_ERR_NULL;
  if (workspace_bytes < need) return T5_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  T5_STEP("adafactor", launch_adafactor_multi(items, n, *cfg, workspace, st));
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
