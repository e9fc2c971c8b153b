// Host-side pieces shared by the C-ABI entry points (block.hip, stack.hip): shape validation, carving of
// the caller's stash and workspace, and the sublayer sequences of the T5.1.1 block.  Everything here
// has internal linkage except the step-timing state, which lives in block.hip.
#pragma once
#include <cmath>
#include <cstring>
#include <string>
#include <vector>
#include "kernels.h"

namespace t5mi {
struct StepRec {
  const char* name;
  hipEvent_t e0, e1;
};
extern bool g_timing;
extern std::vector<StepRec> g_recs;
// Second stream for the weight-gradient GEMMs of a backward pass (t5_wgrad_overlap_enable); null when off.
struct SideStream {
  hipStream_t stream = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
};
extern SideStream g_side;
}  // namespace t5mi

using namespace t5mi;

namespace {

struct Dims {
  int B, S, d, H, dk, F, I;
  int64_t T;
  size_t es;  // bytes per stored element
  int ty;     // IN_F32 / IN_BF16
  int mlp;    // ACT_GELU_TANH / ACT_RELU / ACT_GELU_ERF (the T5_MLP_* values)
  int Sk;     // encoder length of the cross-attention sublayer; 0: block without cross-attention
  int64_t Te; // B * Sk
  float drop;     // dropout rate; 0: none
  uint64_t seed;  // dropout seed
  int det;        // 1: weight and bias-table gradients are summed in a fixed order
};
// Generator parameters of one of the block's dropout sites (off when the rate is 0).
inline DropSite drop_site(const Dims& D, int site) { return make_drop_site(D.seed, site, D.drop); }

int validate_cfg(const t5_block_cfg* c, Dims* o, RelposLut* lut, int enc_seq = 0) {
  if (!c) return T5_ERR_NULL;
  if (c->batch < 1 || c->seq < 1 || c->d_model < 1 || c->n_heads < 1 || c->d_kv < 1 || c->d_ff < 1 || enc_seq < 0)
    return T5_ERR_SHAPE;
  if (c->dtype != T5_F32 && c->dtype != T5_BF16) return T5_ERR_UNSUPPORTED;
  if (c->mlp_kind != T5_MLP_GEGLU_TANH && c->mlp_kind != T5_MLP_RELU && c->mlp_kind != T5_MLP_GEGLU_ERF)
    return T5_ERR_UNSUPPORTED;
  if (!(c->rms_eps >= 0.f) || !std::isfinite(c->attn_scale)) return T5_ERR_SHAPE;
  if (!(c->dropout_rate >= 0.f && c->dropout_rate < 1.f)) return T5_ERR_SHAPE;
  if (c->deterministic != 0 && c->deterministic != 1) return T5_ERR_SHAPE;
  const int64_t T = (int64_t)c->batch * c->seq;
  const int64_t Te = (int64_t)c->batch * enc_seq;
  const int64_t I = (int64_t)c->n_heads * c->d_kv;
  if (T > (1 << 24) || Te > (1 << 24) || I > (1 << 16) || c->d_model > (1 << 16) || c->d_ff > (1 << 18) ||
      c->seq > (1 << 16) || enc_seq > (1 << 16))
    return T5_ERR_UNSUPPORTED;
  if (c->d_model > 8192 || (c->d_model % 8 != 0 && c->d_model > 1024)) return T5_ERR_UNSUPPORTED;
  if (c->dropout_rate > 0.f && T * c->n_heads > ((int64_t)1 << 32)) return T5_ERR_UNSUPPORTED;  // 32-bit row counter
  RelposLut tmp;
  const int rc = relpos_build_lut(c->causal ? 0 : 1, c->num_buckets, c->max_distance, lut ? lut : &tmp);
  if (rc != T5_OK) return rc;
  if (o) {
    o->B = c->batch; o->S = c->seq; o->d = c->d_model; o->H = c->n_heads; o->dk = c->d_kv; o->F = c->d_ff;
    o->I = (int)I; o->T = T;
    o->ty = c->dtype == T5_BF16 ? IN_BF16 : IN_F32;
    o->es = c->dtype == T5_BF16 ? 2 : 4;
    o->Sk = enc_seq; o->Te = Te;
    o->mlp = c->mlp_kind;
    o->drop = c->dropout_rate;
    o->seed = ((uint64_t)c->dropout_seed_hi << 32) | c->dropout_seed_lo;
    o->det = c->deterministic;
    static_assert(T5_MLP_GEGLU_TANH == ACT_GELU_TANH && T5_MLP_RELU == ACT_RELU && T5_MLP_GEGLU_ERF == ACT_GELU_ERF,
                  "the config values are the kernels' activation codes");
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
  // cross-attention sublayer (D.Sk > 0): h is the stream after self-attention, h2 after cross-attention
  float *rx, *lse_x, *h2;
  void *nx, *qx, *kvx, *cx;  // qx [T, I]; kvx [Te, 2I] (k | v per encoder token); cx [T, I]
};
size_t carve_stash(const Dims& D, void* base, Stash* s) {
  Carver cv(base);
  Stash t;
  std::memset(&t, 0, sizeof(t));
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
  if (D.Sk > 0) {
    t.rx = cv.take<float>(D.T * 4);
    t.lse_x = cv.take<float>((size_t)D.B * D.H * D.S * 4);
    t.h2 = cv.take<float>((size_t)D.T * D.d * 4);
    t.nx = cv.take((size_t)D.T * D.d * D.es);
    t.qx = cv.take((size_t)D.T * D.I * D.es);
    t.kvx = cv.take((size_t)D.Te * 2 * D.I * D.es);
    t.cx = cv.take((size_t)D.T * D.I * D.es);
  }
  if (s) *s = t;
  return cv.off;
}

struct FwdWs {
  void *wqkv_t, *wo_t, *wi_t, *woff_t;  // packed transposed weights (bf16 MFMA path)
  void *xq_t, *xkv_t, *xo_t;            // the same for the cross-attention projections
};
size_t carve_fwd(const Dims& D, void* base, FwdWs* w) {
  Carver cv(base);
  FwdWs t;
  std::memset(&t, 0, sizeof(t));
  t.wqkv_t = cv.take((size_t)3 * D.I * D.d * D.es);
  t.wo_t = cv.take((size_t)D.d * D.I * D.es);
  t.wi_t = cv.take((size_t)2 * D.F * D.d * D.es);
  t.woff_t = cv.take((size_t)D.d * D.F * D.es);
  if (D.Sk > 0) {
    t.xq_t = cv.take((size_t)D.I * D.d * D.es);
    t.xkv_t = cv.take((size_t)2 * D.I * D.d * D.es);
    t.xo_t = cv.take((size_t)D.d * D.I * D.es);
  }
  if (w) *w = t;
  return cv.off;
}

// Fork/join of one backward pass.  The weight gradients are leaves of the backward's dependency graph:
// nothing later in the pass reads them.  With a side stream they run beside the chain that carries the
// gradient to the layer's input, filling compute units that chain's smaller kernels leave idle.
// fork_sync() makes the side stream wait for everything launched on the main stream so far (the producers
// of the GEMM's operands, and the clearing of the gradients); fork_join() makes the main stream wait for
// the side stream, before buffers the side GEMMs read are written again (the next layer, the next call).
struct Fork {
  hipStream_t main = nullptr, side = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  bool on = false;
};
inline Fork fork_begin(hipStream_t st, bool allowed) {
  Fork f;
  f.main = st;
  if (!allowed || !t5mi::g_side.stream) return f;
  // a pass that is being recorded into a graph stays on the caller's stream
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) return f;
  f.side = t5mi::g_side.stream; f.ev_fork = t5mi::g_side.ev_fork; f.ev_join = t5mi::g_side.ev_join;
  f.on = true;
  return f;
}
inline hipError_t fork_sync(const Fork& f) {
  if (!f.on) return hipSuccess;
  hipError_t e = hipEventRecord(f.ev_fork, f.main);
  return e != hipSuccess ? e : hipStreamWaitEvent(f.side, f.ev_fork, 0);
}
inline hipError_t fork_join(const Fork& f) {
  if (!f.on) return hipSuccess;
  hipError_t e = hipEventRecord(f.ev_join, f.side);
  return e != hipSuccess ? e : hipStreamWaitEvent(f.main, f.ev_join, 0);
}
inline hipStream_t wgrad_stream(const Fork& f) { return f.on ? f.side : f.main; }
// Joins the side stream on every way out of a backward pass: an error return between fork and join must
// not leave side-stream GEMMs running on buffers the caller is about to reuse.
struct ForkGuard {
  const Fork& f;
  bool done = false;
  explicit ForkGuard(const Fork& fk) : f(fk) {}
  hipError_t join() { done = true; return fork_join(f); }
  ~ForkGuard() { if (!done) (void)fork_join(f); }
};

struct BwdWs {
  Fork fork;
  // set by a stack that launches the weight-gradient GEMMs of all its layers together after the sweep: the
  // layer functions then skip theirs and leave the operands (duw, dh_lp / dh1_lp, dqkv, dqx, dkvx) in place
  bool defer_wgrad = false;
  float *dn, *dh, *dvec, *ddiag, *dg_partial;
  void *dh_lp, *duw, *dc, *dqkv;  // duw: [T][2F], du in columns 0..F-1, dw in F..2F-1
  // cross-attention sublayer: dh/dh_lp hold the gradient of h2, dh1/dh1_lp that of h
  float* dh1;
  void *dh1_lp, *dqx, *dkvx;  // dqx [T, I]; dkvx [Te, 2I]
  // [T, d] each (dropout only): a sublayer's output gradient times its dropout multiplier, one buffer per
  // sublayer (feed-forward, self-attention, cross-attention) so that all three outlive the layer's pass
  void *dmask, *dmask_a, *dmask_x;
  // reproducible mode (D.det): room for the k-slices' partial sums of the largest weight-gradient GEMM of the
  // layer (the GEMMs run one after the other and share it), and for the bias-gradient windows of the
  // attention backward's workgroups
  float *wg_partials, *ddiag_part;
};
size_t wgrad_partials_bytes(const Dims& D);  // defined below, after the GEMM descriptor helpers
size_t carve_bwd(const Dims& D, void* base, BwdWs* w) {
  Carver cv(base);
  BwdWs t = {};
  t.dn = cv.take<float>((size_t)D.T * D.d * 4);
  t.dh = cv.take<float>((size_t)D.T * D.d * 4);
  t.dvec = cv.take<float>((size_t)2 * D.B * D.H * D.S * 4);  // rowsum(dO * O), and the forward's lse rescaled, per query
  t.ddiag = cv.take<float>((size_t)D.H * (2 * D.S - 1) * 4);
  t.dg_partial = cv.take<float>((size_t)rmsnorm_bwd_partial_rows((int)D.T) * D.d * 4);
  t.dh_lp = cv.take(D.ty == IN_BF16 ? (size_t)D.T * D.d * D.es : 0);
  t.duw = cv.take((size_t)D.T * 2 * D.F * D.es);
  t.dc = cv.take((size_t)D.T * D.I * D.es);
  t.dqkv = cv.take((size_t)D.T * 3 * D.I * D.es);
  t.dmask = cv.take(D.drop > 0.f ? (size_t)D.T * D.d * D.es : 0);
  t.dmask_a = cv.take(D.drop > 0.f ? (size_t)D.T * D.d * D.es : 0);
  if (D.Sk > 0) {
    t.dh1 = cv.take<float>((size_t)D.T * D.d * 4);
    t.dh1_lp = cv.take(D.ty == IN_BF16 ? (size_t)D.T * D.d * D.es : 0);
    t.dqx = cv.take((size_t)D.T * D.I * D.es);
    t.dkvx = cv.take((size_t)D.Te * 2 * D.I * D.es);
    t.dmask_x = cv.take(D.drop > 0.f ? (size_t)D.T * D.d * D.es : 0);
  }
  if (D.det && D.ty == IN_BF16) {
    t.wg_partials = cv.take<float>(wgrad_partials_bytes(D));
    AttnDims ad;
    std::memset(&ad, 0, sizeof(ad));
    ad.B = D.B; ad.S = D.S; ad.H = D.H;
    t.ddiag_part = cv.take<float>(D.S % 128 == 0 ? attn_ddiag_part_bytes(ad) : 0);
  }
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

// Room for the partial sums of the layer's largest split weight-gradient GEMM (reproducible mode).
size_t wgrad_partials_bytes(const Dims& D) {
  alignas(16) static const long long dummy[4] = {0, 0, 0, 0};
  const int T = (int)D.T, Te = (int)D.Te;
  size_t need = 0;
  auto probe = [&](int M, int N, int K) {
    GemmDesc g = gemm1(M, N, K, dummy, M, 0, dummy, N, 0, IN_BF16);
    const size_t b = gemm_split_partials_bytes(g, epi(EPI_SPLIT_F32, (void*)dummy, N, IN_F32));
    need = b > need ? b : need;
  };
  probe(D.F, D.d, T);                                   // dWo_ff
  probe(D.d, D.mlp == ACT_RELU ? D.F : 2 * D.F, T);     // dWi0 | dWi1
  probe(D.I, D.d, T);                                   // dWo (and dXo)
  probe(D.d, 3 * D.I, T);                               // dWq | dWk | dWv
  if (D.Sk > 0) {
    probe(D.d, D.I, T);                                 // dXq
    probe(D.d, 2 * D.I, Te);                            // dXk | dXv
  }
  return need;
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
using t5mi::g_timing;
using t5mi::g_recs;
using t5mi::StepRec;

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
  alignas(16) static const long long dummy[4] = {0, 0, 0, 0};  // placeholder operand: passes the 16-byte alignment test
  if (D.mlp == ACT_RELU) {
    GemmDesc g = gemm1((int)D.T, D.F, D.d, dummy, D.d, 1, dummy, D.d, 1, IN_BF16);
    return gemm_mfma_supported(g, epi(EPI_STORE, (void*)dummy, D.F, IN_BF16));
  }
  GemmDesc g = gemm1((int)D.T, 2 * D.F, D.d, dummy, D.d, 1, dummy, D.d, 1, IN_BF16);
  GemmEpi e = epi(EPI_GEGLU_FWD, (void*)dummy, D.F, IN_BF16);
  e.out1 = (void*)dummy; e.out2 = (void*)dummy;
  return gemm_mfma_supported(g, e);
}

// The ungated feed-forward has no wi1.
bool weights_present(const t5_block_weights* w, const Dims& D) {
  return w->ln1_scale && w->wq && w->wk && w->wv && w->wo && w->rel_table && w->ln2_scale && w->wi0 &&
         (w->wi1 || D.mlp == ACT_RELU) && w->wo_ff;
}
bool grads_present(const t5_block_grads* g, const Dims& D) {
  return g->ln1_scale && g->wq && g->wk && g->wv && g->wo && g->rel_table && g->ln2_scale && g->wi0 &&
         (g->wi1 || D.mlp == ACT_RELU) && g->wo_ff;
}

AttnDims self_dims(const t5_block_cfg* cfg, const Dims& D) {
  return AttnDims{D.B, D.S, D.H, D.dk, cfg->causal ? 1 : 0, cfg->attn_scale, D.S, 1, drop_site(D, DROP_ATTN_PROBS)};
}
AttnDims cross_dims(const t5_block_cfg* cfg, const Dims& D) {
  return AttnDims{D.B, D.S, D.H, D.dk, 0, cfg->attn_scale, D.Sk, 0, drop_site(D, DROP_CROSS_PROBS)};
}
AttnIO cross_io(const Dims& D, const Stash& S, const BwdWs* W) {
  AttnIO io;
  std::memset(&io, 0, sizeof(io));
  io.q = S.qx; io.k = S.kvx; io.v = at((const void*)S.kvx, (size_t)D.I, D.es);
  io.ldq = D.I; io.ldkv = 2 * D.I;
  if (W) {
    io.dq = W->dqx; io.dk = W->dkvx; io.dv = at(W->dkvx, (size_t)D.I, D.es);
    io.lddq = D.I; io.lddkv = 2 * D.I;
  }
  return io;
}

// ------------------------------------------------------------------ forward sublayers
// All weight packs (transposes to k-contiguous rows) of the layer in one launch.
int fwd_pack_weights(const Dims& D, const t5_block_weights* w, const t5_cross_weights* xw, const FwdWs& W,
                     hipStream_t st) {
  PackJobs pj;
  std::memset(&pj, 0, sizeof(pj));
  pj.j[0] = PackJob{{w->wq, w->wk, w->wv}, 3, D.d, D.I, 0, W.wqkv_t};
  pj.j[1] = PackJob{{w->wo, nullptr, nullptr}, 1, D.I, D.d, 0, W.wo_t};
  if (D.mlp == ACT_RELU) pj.j[2] = PackJob{{w->wi0, nullptr, nullptr}, 1, D.d, D.F, 0, W.wi_t};
  else pj.j[2] = PackJob{{w->wi0, w->wi1, nullptr}, 2, D.d, D.F, 32, W.wi_t};
  pj.j[3] = PackJob{{w->wo_ff, nullptr, nullptr}, 1, D.F, D.d, 0, W.woff_t};
  pj.count = 4;
  if (xw) {
    pj.j[4] = PackJob{{xw->xq, nullptr, nullptr}, 1, D.d, D.I, 0, W.xq_t};
    pj.j[5] = PackJob{{xw->xk, xw->xv, nullptr}, 2, D.d, D.I, 0, W.xkv_t};
    pj.j[6] = PackJob{{xw->xo, nullptr, nullptr}, 1, D.I, D.d, 0, W.xo_t};
    pj.count = 7;
  }
  T5_STEP("pack_weights", launch_pack_transpose_multi(pj, st));
  return T5_OK;
}

// S.h = x + SelfAttn(RMSNorm(x; ln1_scale))   (float32 residual stream)
// own_table: the layer builds the bias diagonals S.diag from its table; otherwise S.diag already holds
// them (a stack shares one table between its layers).
int fwd_self_attn(const t5_block_cfg* cfg, const Dims& D, const RelposLut& lut, const void* x,
                  const t5_block_weights* w, const Stash& S, const FwdWs& W, bool fused, hipStream_t st,
                  bool own_table = true) {
  const int T = (int)D.T, ty = D.ty;
  const size_t es = D.es;
  const AttnDims ad = self_dims(cfg, D);
  if (own_table) T5_STEP("relpos_diag", launch_relpos_diag(w->rel_table, cfg->dtype, S.diag, D.S, D.H, lut, st));
  T5_STEP("rmsnorm_fwd", launch_rmsnorm_fwd(x, ty, w->ln1_scale, S.n1, ty, S.r1, T, D.d, cfg->rms_eps, st));
  if (fused) {
    GemmDesc g = gemm1(T, 3 * D.I, D.d, S.n1, D.d, 1, W.wqkv_t, D.d, 1, ty);
    T5_STEP("gemm_qkv", run_gemm(g, epi(EPI_STORE, S.qkv, 3 * D.I, ty), st));
  } else {
    const void* ws3[3] = {w->wq, w->wk, w->wv};
    for (int j = 0; j < 3; ++j) {
      GemmDesc g = gemm1(T, D.I, D.d, S.n1, D.d, 1, ws3[j], D.I, 0, ty);
      T5_STEP("gemm_qkv", run_gemm(g, epi(EPI_STORE, at(S.qkv, (size_t)j * D.I, es), 3 * D.I, ty), st));
    }
  }
  const AttnIO io = attn_io_packed(S.qkv, nullptr, D.I, es);
  if (ty == IN_BF16 && attn_mfma_supported(ad))
    T5_STEP("attn_fwd", launch_attn_fwd_mfma(io, S.diag, S.c, S.lse, ad, st));
  else
    T5_STEP("attn_fwd", launch_attn_fwd_simple(io, ty, S.diag, S.c, S.lse, ad, st));
  GemmDesc g = fused ? gemm1(T, D.d, D.I, S.c, D.I, 1, W.wo_t, D.I, 1, ty)
                     : gemm1(T, D.d, D.I, S.c, D.I, 1, w->wo, D.d, 0, ty);
  GemmEpi e = epi(EPI_RESID, S.h, D.d, IN_F32);
  e.aux0 = x; e.aux_type = ty; e.drop = drop_site(D, DROP_ATTN_OUT);
  T5_STEP("gemm_o", run_gemm(g, e, st));
  return T5_OK;
}

// S.h2 = S.h + CrossAttn(RMSNorm(S.h; lnx_scale), enc)
int fwd_cross_attn(const t5_block_cfg* cfg, const Dims& D, const void* enc, const t5_cross_weights* xw,
                   const Stash& S, const FwdWs& W, bool fused, hipStream_t st) {
  const int T = (int)D.T, Te = (int)D.Te, ty = D.ty;
  const size_t es = D.es;
  const AttnDims ad = cross_dims(cfg, D);
  T5_STEP("rmsnorm_fwd", launch_rmsnorm_fwd(S.h, IN_F32, xw->lnx_scale, S.nx, ty, S.rx, T, D.d, cfg->rms_eps, st));
  if (fused) {
    GemmDesc gq = gemm1(T, D.I, D.d, S.nx, D.d, 1, W.xq_t, D.d, 1, ty);
    T5_STEP("gemm_xq", run_gemm(gq, epi(EPI_STORE, S.qx, D.I, ty), st));
    GemmDesc gkv = gemm1(Te, 2 * D.I, D.d, enc, D.d, 1, W.xkv_t, D.d, 1, ty);
    T5_STEP("gemm_xkv", run_gemm(gkv, epi(EPI_STORE, S.kvx, 2 * D.I, ty), st));
  } else {
    GemmDesc gq = gemm1(T, D.I, D.d, S.nx, D.d, 1, xw->xq, D.I, 0, ty);
    T5_STEP("gemm_xq", run_gemm(gq, epi(EPI_STORE, S.qx, D.I, ty), st));
    const void* ws2[2] = {xw->xk, xw->xv};
    for (int j = 0; j < 2; ++j) {
      GemmDesc g = gemm1(Te, D.I, D.d, enc, D.d, 1, ws2[j], D.I, 0, ty);
      T5_STEP("gemm_xkv", run_gemm(g, epi(EPI_STORE, at(S.kvx, (size_t)j * D.I, es), 2 * D.I, ty), st));
    }
  }
  const AttnIO io = cross_io(D, S, nullptr);
  if (ty == IN_BF16 && attn_mfma_supported(ad))
    T5_STEP("xattn_fwd", launch_attn_fwd_mfma(io, nullptr, S.cx, S.lse_x, ad, st));
  else
    T5_STEP("xattn_fwd", launch_attn_fwd_simple(io, ty, nullptr, S.cx, S.lse_x, ad, st));
  GemmDesc g = fused ? gemm1(T, D.d, D.I, S.cx, D.I, 1, W.xo_t, D.I, 1, ty)
                     : gemm1(T, D.d, D.I, S.cx, D.I, 1, xw->xo, D.d, 0, ty);
  GemmEpi e = epi(EPI_RESID, S.h2, D.d, IN_F32);
  e.aux0 = S.h; e.aux_type = IN_F32; e.drop = drop_site(D, DROP_CROSS_OUT);
  T5_STEP("gemm_xo", run_gemm(g, e, st));
  return T5_OK;
}

// y = hin + MLP(RMSNorm(hin; ln2_scale))   hin: float32 residual stream
int fwd_mlp(const t5_block_cfg* cfg, const Dims& D, const float* hin, const t5_block_weights* w, const Stash& S,
            const FwdWs& W, bool fused, void* y, hipStream_t st) {
  const int T = (int)D.T, ty = D.ty;
  T5_STEP("rmsnorm_fwd", launch_rmsnorm_fwd(hin, IN_F32, w->ln2_scale, S.n2, ty, S.r2, T, D.d, cfg->rms_eps, st));
  if (D.mlp == ACT_RELU) {  // a = max(n2 Wi0, 0); the backward reads the mask off a itself
    GemmDesc g = fused ? gemm1(T, D.F, D.d, S.n2, D.d, 1, W.wi_t, D.d, 1, ty)
                       : gemm1(T, D.F, D.d, S.n2, D.d, 1, w->wi0, D.F, 0, ty);
    GemmEpi e = epi(EPI_STORE, S.a, D.F, ty);
    e.act = ACT_RELU; e.drop = drop_site(D, DROP_MLP_HIDDEN);
    T5_STEP("gemm_wi_relu", run_gemm(g, e, st));
  } else if (fused) {
    GemmDesc g = gemm1(T, 2 * D.F, D.d, S.n2, D.d, 1, W.wi_t, D.d, 1, ty);
    GemmEpi e = epi(EPI_GEGLU_FWD, S.gp, D.F, ty);
    e.out1 = S.gl; e.out2 = S.a; e.act = D.mlp; e.drop = drop_site(D, DROP_MLP_HIDDEN);
    if (!gemm_mfma_supported(g, e)) return T5_ERR_UNSUPPORTED;
    T5_STEP("gemm_wi_geglu", launch_gemm_mfma(g, e, st));
  } else {
    GemmDesc g0 = gemm1(T, D.F, D.d, S.n2, D.d, 1, w->wi0, D.F, 0, ty);
    T5_STEP("gemm_wi", run_gemm(g0, epi(EPI_STORE, S.gp, D.F, ty), st));
    GemmDesc g1 = gemm1(T, D.F, D.d, S.n2, D.d, 1, w->wi1, D.F, 0, ty);
    T5_STEP("gemm_wi", run_gemm(g1, epi(EPI_STORE, S.gl, D.F, ty), st));
    T5_STEP("geglu_fwd", launch_geglu_fwd(S.gp, S.gl, S.a, ty, (int64_t)D.T * D.F, D.mlp,
                                          drop_site(D, DROP_MLP_HIDDEN), D.F, st));
  }
  GemmDesc g = fused ? gemm1(T, D.d, D.F, S.a, D.F, 1, W.woff_t, D.F, 1, ty)
                     : gemm1(T, D.d, D.F, S.a, D.F, 1, w->wo_ff, D.d, 0, ty);
  GemmEpi e = epi(EPI_RESID, y, D.d, ty);
  e.aux0 = hin; e.aux_type = IN_F32; e.drop = drop_site(D, DROP_MLP_OUT);
  T5_STEP("gemm_wo", run_gemm(g, e, st));
  return T5_OK;
}

// ------------------------------------------------------------------ backward sublayers
// One launch clears what later kernels add into: the weight gradients (split-k partial sums; kept
// when the caller accumulates) and the bias-gradient diagonals of the fused attention.
int bwd_zero(const Dims& D, const t5_block_grads* dw, const t5_cross_grads* dxw, float* ddiag, bool acc,
             hipStream_t st) {
  ZeroList z;
  std::memset(&z, 0, sizeof(z));
  auto add = [&](float* p, int64_t n) { z.p[z.count] = p; z.n[z.count] = n; ++z.count; };
  if (ddiag) add(ddiag, (int64_t)D.H * (2 * D.S - 1));
  if (!acc) {
    const int64_t dI = (int64_t)D.d * D.I, dF = (int64_t)D.d * D.F;
    add(dw->wq, dI); add(dw->wk, dI); add(dw->wv, dI); add(dw->wo, dI);
    add(dw->wi0, dF); add(dw->wo_ff, dF);
    if (D.mlp != ACT_RELU) add(dw->wi1, dF);
    if (dxw) { add(dxw->xq, dI); add(dxw->xk, dI); add(dxw->xv, dI); add(dxw->xo, dI); }
  }
  static_assert(ZERO_MAX >= 12, "ddiag + 7 block gradients + 4 cross-attention gradients");
  if (z.count > 0) T5_STEP("zero_grads", launch_zero_f32(z, st));
  return T5_OK;
}

// Given dy: W.dh (float32) and, for bf16, W.dh_lp = dy + RMSNormBwd(hin, ln2_scale, dn2); weight
// gradients of the MLP and of ln2_scale.
int bwd_mlp(const Dims& D, const void* dy, const float* hin, const t5_block_weights* w, const Stash& S,
            const BwdWs& W, const t5_block_grads* dw, int acc, hipStream_t st) {
  const int T = (int)D.T, ty = D.ty;
  const size_t es = D.es;
  void* du_p = W.duw;
  void* dw_p = at(W.duw, (size_t)D.F, es);
  const void* dy_in = dy;  // the residual branch takes dy itself, the sublayer dy times its output multiplier
  if (D.drop > 0.f) {
    T5_STEP("dropout_dy", launch_dropout_apply(drop_site(D, DROP_MLP_OUT), dy, W.dmask, ty, T, D.d, st));
    dy = W.dmask;
  }
  if (!W.defer_wgrad) {  // dWo_ff = a^T dy
    T5_TRY(fork_sync(W.fork));
    hipStream_t st = wgrad_stream(W.fork);
    GemmDesc g = gemm1(D.F, D.d, T, S.a, D.F, 0, dy, D.d, 0, ty);
    GemmEpi e = epi(EPI_SPLIT_F32, dw->wo_ff, D.d, IN_F32);
    e.accumulate = 1; e.aux0 = W.wg_partials;
    T5_STEP("gemm_dwo_ff", run_gemm(g, e, st));
  }
  if (D.mlp == ACT_RELU) {
    {  // du = (dy Wo_ff^T) where a > 0
      GemmDesc g = gemm1(T, D.F, D.d, dy, D.d, 1, w->wo_ff, D.d, 1, ty);
      GemmEpi e = epi(EPI_RESID, du_p, D.F, ty);
      e.aux0 = S.a; e.aux_type = ty; e.aux_mask = 1; e.drop = drop_site(D, DROP_MLP_HIDDEN);
      T5_STEP("gemm_da_relu_bwd", run_gemm(g, e, st));
    }
    if (!W.defer_wgrad) {  // dWi0 = n2^T du
      T5_TRY(fork_sync(W.fork));
      hipStream_t st = wgrad_stream(W.fork);
      GemmDesc g = gemm1(D.d, D.F, T, S.n2, D.d, 0, du_p, D.F, 0, ty);
      GemmEpi e = epi(EPI_SPLIT_F32, dw->wi0, D.F, IN_F32);
      e.accumulate = 1; e.aux0 = W.wg_partials;
      T5_STEP("gemm_dwi", run_gemm(g, e, st));
    }
    {  // dn2 = du Wi0^T
      GemmDesc g = gemm1(T, D.d, D.F, du_p, D.F, 1, w->wi0, D.F, 1, ty);
      T5_STEP("gemm_dn2", run_gemm(g, epi(EPI_STORE, W.dn, D.d, IN_F32), st));
    }
  } else {
    {  // da = dy Wo_ff^T, fused with the gated-GELU backward: du = da w gelu'(u), dw = da gelu(u)
      GemmDesc g = gemm1(T, D.F, D.d, dy, D.d, 1, w->wo_ff, D.d, 1, ty);
      GemmEpi e = epi(EPI_GEGLU_BWD, du_p, 2 * D.F, ty);
      e.out1 = dw_p; e.aux0 = S.gp; e.aux1 = S.gl; e.aux_type = ty; e.ld_aux = D.F;
      T5_STEP("gemm_da_geglu_bwd", run_gemm(g, e, st));
    }
    if (!W.defer_wgrad) {  // dWi0 | dWi1 = n2^T [du | dw]
      T5_TRY(fork_sync(W.fork));
      hipStream_t st = wgrad_stream(W.fork);
      GemmDesc g = gemm1(D.d, 2 * D.F, T, S.n2, D.d, 0, du_p, 2 * D.F, 0, ty);
      GemmEpi e = epi(EPI_SPLIT_F32, dw->wi0, D.F, IN_F32);
      e.out1 = dw->wi1; e.split_n = D.F; e.accumulate = 1; e.aux0 = W.wg_partials;
      T5_STEP("gemm_dwi", run_gemm(g, e, st));
    }
    {  // dn2 = du Wi0^T + dw Wi1^T
      GemmDesc g = gemm1(T, D.d, D.F, du_p, 2 * D.F, 1, w->wi0, D.F, 1, ty);
      g.nseg = 2;
      g.seg[1] = GemmSeg{dw_p, w->wi1, 2 * D.F, D.F, D.F};
      T5_STEP("gemm_dn2", run_gemm(g, epi(EPI_STORE, W.dn, D.d, IN_F32), st));
    }
  }
  T5_STEP("rmsnorm_bwd", launch_rmsnorm_bwd(hin, IN_F32, w->ln2_scale, ty, S.r2, W.dn, dy_in, ty, W.dh,
                            ty == IN_BF16 ? W.dh_lp : nullptr, ty, dw->ln2_scale, W.dg_partial, acc, T, D.d,
                            st));
  return T5_OK;
}

// Given W.dh / W.dh_lp (gradient of h2): W.dh1 / W.dh1_lp (gradient of h), denc, and the weight
// gradients of the cross-attention sublayer.  denc is written in the storage type, or (denc_f32) as
// float32, optionally added to what it holds (a stack sums the encoder-output gradients of its layers).
int bwd_cross_attn(const t5_block_cfg* cfg, const Dims& D, const void* enc, const t5_cross_weights* xw,
                   const Stash& S, const BwdWs& W, void* denc, const t5_cross_grads* dxw, int acc, hipStream_t st,
                   bool denc_f32 = false, bool denc_add = false) {
  const int T = (int)D.T, Te = (int)D.Te, ty = D.ty;
  const size_t es = D.es;
  const AttnDims ad = cross_dims(cfg, D);
  const void* dh_op = ty == IN_BF16 ? (const void*)W.dh_lp : (const void*)W.dh;
  if (D.drop > 0.f) {
    T5_STEP("dropout_dh", launch_dropout_apply(drop_site(D, DROP_CROSS_OUT), dh_op, W.dmask_x, ty, T, D.d, st));
    dh_op = W.dmask_x;
  }
  if (!W.defer_wgrad) {  // dXo = cx^T dh2
    T5_TRY(fork_sync(W.fork));
    hipStream_t st = wgrad_stream(W.fork);
    GemmDesc g = gemm1(D.I, D.d, T, S.cx, D.I, 0, dh_op, D.d, 0, ty);
    GemmEpi e = epi(EPI_SPLIT_F32, dxw->xo, D.d, IN_F32);
    e.accumulate = 1; e.aux0 = W.wg_partials;
    T5_STEP("gemm_dxo", run_gemm(g, e, st));
  }
  {  // dcx = dh2 Xo^T
    GemmDesc g = gemm1(T, D.I, D.d, dh_op, D.d, 1, xw->xo, D.d, 1, ty);
    T5_STEP("gemm_dcx", run_gemm(g, epi(EPI_STORE, W.dc, D.I, ty), st));
  }
  const AttnIO io = cross_io(D, S, &W);
  if (ty == IN_BF16 && attn_mfma_supported(ad)) {
    T5_STEP("xattn_bwd_dq", launch_attn_bwd_mfma(io, S.cx, W.dc, nullptr, S.lse_x, W.dvec, nullptr, ad, 1, 1, st));
    T5_STEP("xattn_bwd_dkv", launch_attn_bwd_mfma(io, S.cx, W.dc, nullptr, S.lse_x, W.dvec, nullptr, ad, 1, 2, st));
  } else {
    T5_STEP("xattn_bwd", launch_attn_bwd_simple(io, S.cx, W.dc, ty, nullptr, S.lse_x, W.dvec, nullptr, ad, 0, st));
  }
  if (!W.defer_wgrad) {  // dXq = nx^T dq
    T5_TRY(fork_sync(W.fork));
    hipStream_t st = wgrad_stream(W.fork);
    GemmDesc g = gemm1(D.d, D.I, T, S.nx, D.d, 0, W.dqx, D.I, 0, ty);
    GemmEpi e = epi(EPI_SPLIT_F32, dxw->xq, D.I, IN_F32);
    e.accumulate = 1; e.aux0 = W.wg_partials;
    T5_STEP("gemm_dxq", run_gemm(g, e, st));
  }
  if (!W.defer_wgrad) {  // dXk | dXv = enc^T [dk | dv]   (ordered after dXq on the side stream: no new fork point needed)
    hipStream_t st = wgrad_stream(W.fork);
    GemmDesc g = gemm1(D.d, 2 * D.I, Te, enc, D.d, 0, W.dkvx, 2 * D.I, 0, ty);
    GemmEpi e = epi(EPI_SPLIT_F32, dxw->xk, D.I, IN_F32);
    e.out1 = dxw->xv; e.split_n = D.I; e.accumulate = 1; e.aux0 = W.wg_partials;
    T5_STEP("gemm_dxkv", run_gemm(g, e, st));
  }
  {  // denc = dk Xk^T + dv Xv^T
    GemmDesc g = gemm1(Te, D.d, D.I, W.dkvx, 2 * D.I, 1, xw->xk, D.I, 1, ty);
    g.nseg = 2;
    g.seg[1] = GemmSeg{at(W.dkvx, (size_t)D.I, es), xw->xv, 2 * D.I, D.I, D.I};
    GemmEpi e = epi(denc_add ? EPI_RESID : EPI_STORE, denc, D.d, denc_f32 ? IN_F32 : ty);
    if (denc_add) { e.aux0 = denc; e.aux_type = denc_f32 ? IN_F32 : ty; }  // in place: each element is read, then written, by one lane
    T5_STEP("gemm_denc", run_gemm(g, e, st));
  }
  {  // dnx = dq Xq^T
    GemmDesc g = gemm1(T, D.d, D.I, W.dqx, D.I, 1, xw->xq, D.I, 1, ty);
    T5_STEP("gemm_dnx", run_gemm(g, epi(EPI_STORE, W.dn, D.d, IN_F32), st));
  }
  // dh1 = dh2 + RMSNormBwd(h, lnx_scale, dnx)
  T5_STEP("rmsnorm_bwd", launch_rmsnorm_bwd(S.h, IN_F32, xw->lnx_scale, ty, S.rx, W.dn, W.dh, IN_F32, W.dh1,
                            ty == IN_BF16 ? W.dh1_lp : nullptr, ty, dxw->lnx_scale, W.dg_partial, acc, T, D.d,
                            st));
  return T5_OK;
}

// Given dh (float32) and dh_lp (bf16 copy, bf16 blocks) = gradient of S.h: dx and the weight
// gradients of the self-attention sublayer.
int bwd_self_attn(const t5_block_cfg* cfg, const Dims& D, const RelposLut& lut, const void* x, const float* dh,
                  const void* dh_lp, const t5_block_weights* w, const Stash& S, const BwdWs& W, bool attn_mfma,
                  int far, void* dx, const t5_block_grads* dw, int acc, hipStream_t st, bool own_table = true) {
  const int T = (int)D.T, ty = D.ty;
  const size_t es = D.es;
  const AttnDims ad = self_dims(cfg, D);
  const void* dh_op = ty == IN_BF16 ? dh_lp : (const void*)dh;
  if (D.drop > 0.f) {
    T5_STEP("dropout_dh", launch_dropout_apply(drop_site(D, DROP_ATTN_OUT), dh_op, W.dmask_a, ty, T, D.d, st));
    dh_op = W.dmask_a;
  }
  if (!W.defer_wgrad) {  // dWo = c^T dh
    T5_TRY(fork_sync(W.fork));
    hipStream_t st = wgrad_stream(W.fork);
    GemmDesc g = gemm1(D.I, D.d, T, S.c, D.I, 0, dh_op, D.d, 0, ty);
    GemmEpi e = epi(EPI_SPLIT_F32, dw->wo, D.d, IN_F32);
    e.accumulate = 1; e.aux0 = W.wg_partials;
    T5_STEP("gemm_dwo", run_gemm(g, e, st));
  }
  {  // dc = dh Wo^T
    GemmDesc g = gemm1(T, D.I, D.d, dh_op, D.d, 1, w->wo, D.d, 1, ty);
    T5_STEP("gemm_dc", run_gemm(g, epi(EPI_STORE, W.dc, D.I, ty), st));
  }
  const AttnIO io = attn_io_packed(S.qkv, W.dqkv, D.I, es);
  if (attn_mfma) {
    T5_STEP("attn_bwd_dq", launch_attn_bwd_mfma(io, S.c, W.dc, S.diag, S.lse, W.dvec, W.ddiag, ad, far, 1, st,
                                                W.ddiag_part));
    T5_STEP("attn_bwd_dkv", launch_attn_bwd_mfma(io, S.c, W.dc, S.diag, S.lse, W.dvec, W.ddiag, ad, far, 2, st));
  } else {
    T5_STEP("attn_bwd", launch_attn_bwd_simple(io, S.c, W.dc, ty, S.diag, S.lse, W.dvec, W.ddiag, ad,
                                               own_table ? 1 : 0, st));
  }
  // a stack with a shared table keeps adding into W.ddiag over its layers and folds it once at the end
  if (own_table)
    T5_STEP("relpos_diag_bwd", launch_relpos_diag_bwd(W.ddiag, dw->rel_table, D.S, D.H, cfg->num_buckets, lut, acc, st));
  if (!W.defer_wgrad) {  // dWq | dWk | dWv = n1^T dqkv
    T5_TRY(fork_sync(W.fork));
    hipStream_t st = wgrad_stream(W.fork);
    GemmDesc g = gemm1(D.d, 3 * D.I, T, S.n1, D.d, 0, W.dqkv, 3 * D.I, 0, ty);
    GemmEpi e = epi(EPI_SPLIT_F32, dw->wq, D.I, IN_F32);
    e.out1 = dw->wk; e.out2 = dw->wv; e.split_n = D.I; e.accumulate = 1; e.aux0 = W.wg_partials;
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
  T5_STEP("rmsnorm_bwd", launch_rmsnorm_bwd(x, ty, w->ln1_scale, ty, S.r1, W.dn, dh, IN_F32,
                            ty == IN_F32 ? (float*)dx : nullptr, ty == IN_BF16 ? dx : nullptr, ty, dw->ln1_scale,
                            W.dg_partial, acc, T, D.d, st));
  return T5_OK;
}

#define T5_SUB(expr)              \
  do {                            \
    const int rc_ = (expr);       \
    if (rc_ != T5_OK) return rc_; \
  } while (0)

}  // namespace
