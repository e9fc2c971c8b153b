// Internal launcher interface between the C-ABI host layer (block.hip) and the kernel files.
// Every launcher enqueues on `st` and returns the hipGetLastError() of its launches.
#pragma once
#include "common.h"

namespace t5mi {

// ------------------------------------------------------------------ relative positions
// Fills `lut` for (bidirectional, num_buckets, max_distance); returns a T5_* status.
int relpos_build_lut(int bidirectional, int num_buckets, int max_distance, RelposLut* lut);
hipError_t launch_relpos_bucket(const int32_t* rel_pos, int32_t* out, int64_t n, const RelposLut& lut,
                                hipStream_t st);
// diag[h][delta + S - 1] = table[bucket(delta)][h] for delta = key - query in [-(S-1), S-1]; float32.
hipError_t launch_relpos_diag(const void* table, int dtype, float* diag, int S, int H,
                              const RelposLut& lut, hipStream_t st);
// dtable[c][h] (+)= sum over delta with bucket(delta) == c of ddiag[h][delta + S - 1]
hipError_t launch_relpos_diag_bwd(const float* ddiag, float* dtable, int S, int H, int num_buckets,
                                  const RelposLut& lut, int accumulate, hipStream_t st);

// ------------------------------------------------------------------ RMSNorm
enum { IN_F32 = 0, IN_BF16 = 1 };
// n = x * r * g, r = rsqrt(mean(x^2) + eps).  x: [T,d] of x_type; g, n of out_type; r: [T] float32.
hipError_t launch_rmsnorm_fwd(const void* x, int x_type, const void* g, void* n, int out_type, float* r,
                              int T, int d, float eps, hipStream_t st);
// dx_total = resid + r * (dn*g - xh * mean(dn*g*xh)),  xh = x*r;  dg (+)= sum_T dn*xh.
// x of x_type; g of g_type; dn float32; resid of resid_type (nullable: no residual term); outputs: out_f32 (nullable),
// out_lp (nullable, lp_type).  dg_partial: workspace float[rmsnorm_bwd_partial_rows(T) * d].
int rmsnorm_bwd_partial_rows(int T);
hipError_t launch_rmsnorm_bwd(const void* x, int x_type, const void* g, int g_type, const float* r,
                              const float* dn, const void* resid, int resid_type, float* out_f32,
                              void* out_lp, int lp_type, float* dg, float* dg_partial, int accumulate,
                              int T, int d, hipStream_t st);

// ------------------------------------------------------------------ GEMM
// C[m,n] = sum over segments s, k < K_s of A_s(m,k) * B_s(n,k), float32 accumulation.
// a_kc: A_s(m,k) = A[m*lda + k], else A[k*lda + m].  b_kc: B_s(n,k) = B[n*ldb + k], else B[k*ldb + n].
struct GemmSeg {
  const void* A;
  const void* B;
  int lda, ldb, K;
};
enum EpiKind {
  EPI_STORE = 0,      // out0[m*ld0 + n] = acc                    (out_type)
  EPI_RESID = 1,      // out0[m*ld0 + n] = acc + aux0[m*ld0 + n]  (aux0 of aux_type)
  // Gated GELU, a = gelu(u) * w.  The forward saves the two factors the backward needs instead of
  // u and w themselves: gp = w * gelu'(u) and gl = gelu(u), so that du = da * gp and dw = da * gl.
  EPI_GEGLU_FWD = 2,  // MFMA path only: B rows interleave wi0/wi1 in groups of 32; out0 = gp, out1 = gl, out2 = a
  EPI_GEGLU_BWD = 3,  // acc = da; reads gp = aux0, gl = aux1; out0 = du, out1 = dw   (all ld0)
  EPI_SPLIT_F32 = 4   // float32 out; column n goes to outs[n / split_n][m*ld0 + n % split_n]; += if accumulate
};
struct GemmEpi {
  int kind;
  void* out0;
  void* out1;
  void* out2;
  // EPI_SPLIT_F32 with a split reduction (MFMA kernel only) reads no auxiliary operand and uses aux0 for
  // something else: when it is set, the k-slices write their partial sums to aux0[slice][m][n] (float32,
  // M x N each, at least gemm_split_partials_bytes()) and a second launch adds the slices up in a fixed order --
  // bit-reproducible, where the default meets in float atomics on the output.
  const void* aux0;
  const void* aux1;
  int ld0;       // leading dimension of out0/out1/out2
  int ld_aux;    // leading dimension of aux0/aux1 (0: same as ld0)
  int out_type;  // IN_F32 / IN_BF16 for out0/out1/out2
  int aux_type;
  int split_n;
  int accumulate;
  int act;       // EPI_STORE: ACT_RELU stores max(acc, 0); EPI_GEGLU_FWD: ACT_GELU_TANH or ACT_GELU_ERF
  int aux_mask;  // EPI_RESID: != 0 stores acc where aux0 > 0 and 0 elsewhere instead of acc + aux0
  // Dropout of the GEMM's result (row = m, column = n; for EPI_GEGLU_FWD column = hidden unit), when drop.on:
  // EPI_RESID stores aux0 + acc * M; EPI_STORE stores act(acc) * M; EPI_GEGLU_FWD multiplies all three
  // outputs by M (so that the saved factors already carry the mask for the backward); with aux_mask
  // the kept value is acc * drop.scale (aux0 is then a masked, rescaled activation).
  DropSite drop;
};
struct GemmDesc {
  int M, N, nseg;
  GemmSeg seg[3];
  int a_kc, b_kc;
  int in_type;  // element type of A and B
  // Several problems of one shape in one launch (EPI_SPLIT_F32 with accumulate, one segment, MFMA kernel only):
  // groups is a DEVICE array of ngroups x GEMM_GROUP_PTRS pointers {A, B, out0, out1, out2}, which replace
  // seg[0].A / .B and the epilogue's outputs for the workgroups of that problem.  ngroups <= 1: one problem.
  const void* const* groups;
  int ngroups;
};
constexpr int GEMM_GROUP_PTRS = 5;
// dst[i] = ptrs[i] for i < n: builds such a table (or any other) in device memory from host values, by kernel
// (no host-to-device copy: callers may be recording a graph).
hipError_t launch_fill_ptrs(const void* const* ptrs, int n, const void** dst, hipStream_t st);
// Simple LDS-tiled FMA kernel: any shape, float32 or bf16 inputs.  Reference-grade speed.
hipError_t launch_gemm_simple(const GemmDesc& g, const GemmEpi& e, hipStream_t st);
// bf16 MFMA kernel.  Requires in_type == IN_BF16, every K % 64 == 0, lda/ldb % 8 == 0, N % 64 == 0
// and 16-byte aligned pointers; gemm_mfma_supported() checks this.
bool gemm_mfma_supported(const GemmDesc& g, const GemmEpi& e);
hipError_t launch_gemm_mfma(const GemmDesc& g, const GemmEpi& e, hipStream_t st);
// Bytes of the partial-sum buffer (GemmEpi::aux0) that launch_gemm_mfma would use for this EPI_SPLIT_F32 problem (0: no split).
size_t gemm_split_partials_bytes(const GemmDesc& g, const GemmEpi& e);

// Sets up to 12 float arrays to zero in one launch (the weight gradients, before the split-k GEMMs add
// their partial sums into them, and the bias-gradient diagonals).
constexpr int ZERO_MAX = 12;
struct ZeroList {
  float* p[ZERO_MAX];
  int64_t n[ZERO_MAX];
  int count;
};
hipError_t launch_zero_f32(const ZeroList& z, hipStream_t st);

// Transpose-pack for the forward weights (bf16): dst[n][k] = src_j[k][n'] for the concatenation of
// nsrc matrices [K, n_each] along n.  interleave > 0: packed row n maps to source
// (n / interleave) % nsrc and column (n / (interleave*nsrc)) * interleave + n % interleave.
hipError_t launch_pack_transpose_bf16(const void* const* srcs, int nsrc, int K, int n_each, void* dst,
                                      int interleave, hipStream_t st);
// Up to eight such packs in one launch.
struct PackJob {
  const void* src[3];
  int nsrc, K, n_each, interleave;
  void* dst;
};
struct PackJobs {
  PackJob j[8];
  int count;
};
hipError_t launch_pack_transpose_multi(const PackJobs& jobs, hipStream_t st);

// ------------------------------------------------------------------ elementwise gated GELU (simple path)
// a = gelu(u) * w; then overwrites u with w * gelu'(u) and w with gelu(u) (the saved backward factors).
// With drop.on all three also carry the dropout multiplier of element (i / cols, i % cols).
hipError_t launch_geglu_fwd(void* u, void* w, void* a, int type, int64_t n, int act, const DropSite& drop, int cols,
                            hipStream_t st);

// ------------------------------------------------------------------ attention
// Queries: S per batch element; keys/values: Sk per batch element (Sk == S for self-attention).
// bias: add the relative-position bias diag[h][j - i + S - 1] (needs Sk == S); causal needs Sk == S.
struct AttnDims {
  int B, S, H, dk;
  int causal;
  float scale;
  int Sk;
  int bias;
  DropSite drop;  // dropout of the probabilities; row = (b*H + h)*S + i, column = j
};
// Operand placement.  Row (b*S + i) of q / dq starts at q + row*ldq, row (b*Sk + j) of k, v / dk, dv at
// k + row*ldkv; head h occupies channels h*dk .. h*dk + dk - 1 of a row.  Element counts, not bytes.
struct AttnIO {
  const void *q, *k, *v;
  int ldq, ldkv;
  void *dq, *dk, *dv;
  int lddq, lddkv;
};
// q | k | v packed per token: qkv [T, 3*I], dqkv likewise (either may be null when unused).
inline AttnIO attn_io_packed(const void* qkv, void* dqkv, int I, size_t es) {
  AttnIO io;
  io.q = qkv; io.k = (const char*)qkv + (size_t)I * es; io.v = (const char*)qkv + (size_t)2 * I * es;
  io.ldq = io.ldkv = 3 * I;
  io.dq = dqkv; io.dk = dqkv ? (char*)dqkv + (size_t)I * es : nullptr;
  io.dv = dqkv ? (char*)dqkv + (size_t)2 * I * es : nullptr;
  io.lddq = io.lddkv = 3 * I;
  return io;
}
// c: [B*S, H*dk].  lse: [B,H,S] float32.  diag: [H, 2S-1] (unused without bias).
hipError_t launch_attn_fwd_simple(const AttnIO& io, int type, const float* diag, void* c, float* lse,
                                  const AttnDims& a, hipStream_t st);
// dc: [B*S, H*dk] gradient of c.  Writes dq, dk, dv, dvec [B,H,S] (scratch) and, with bias, adds the
// bias gradient into ddiag [H, 2S-1] float32 (cleared first when zero_ddiag is set).
hipError_t launch_attn_bwd_simple(const AttnIO& io, const void* c, const void* dc, int type,
                                  const float* diag, const float* lse, float* dvec, float* ddiag,
                                  const AttnDims& a, int zero_ddiag, hipStream_t st);
bool attn_mfma_supported(const AttnDims& a);
hipError_t launch_attn_fwd_mfma(const AttnIO& io, const float* diag, void* c, float* lse, const AttnDims& a,
                                hipStream_t st);
// Whether the backward kernels take this problem with `far` (smallest distance in the saturated last
// bucket); otherwise the simple backward is used (same saved tensors).
bool attn_bwd_mfma_fits(const AttnDims& a, int far);
// phase 1: dq, the per-query scratch and the bias-gradient diagonals, ADDED into ddiag (the caller clears
// it); phase 2: dk, dv (reads the scratch, so it runs after phase 1).  dvec here is 2 x [B,H,S] floats:
// -rowsum(dO * O), then -lse / scale, the two per-query constants the dk/dv kernel stages by DMA.
// ddiag_part (phase 1, with bias; nullable): when given, at least attn_ddiag_part_bytes(); the workgroups then
// write their bias-gradient windows there and a second kernel adds them into ddiag in a fixed order
// (bit-reproducible) instead of meeting in float atomics.
size_t attn_ddiag_part_bytes(const AttnDims& a);
hipError_t launch_attn_bwd_mfma(const AttnIO& io, const void* c, const void* dc, const float* diag,
                                const float* lse, float* dvec, float* ddiag, const AttnDims& a, int far,
                                int phase, hipStream_t st, float* ddiag_part = nullptr);

// ------------------------------------------------------------------ ends of the layer stack
// x[r, :] = E[tokens[r], :] (storage type); ids outside [0, vocab) are clamped into it.
hipError_t launch_embed_fwd(const int32_t* tokens, const void* E, void* x, int type, int64_t rows, int d, int vocab,
                            hipStream_t st);
// dE[tokens[r], :] += dx[r, :]; the caller clears dE.  ordered == 0: float32 atomics, one wave per token row.
// ordered != 0: one wave per vocabulary row, which adds the rows of its tokens in position order (bit-reproducible;
// every wave scans all the tokens).
hipError_t launch_embed_bwd(const int32_t* tokens, const void* dx, int type, float* dE, int64_t rows, int d,
                            int vocab, int ordered, hipStream_t st);
// *n_valid = number of rows with 0 <= target < vocab, as a float.
hipError_t launch_xent_count(const int32_t* targets, int64_t rows, int vocab, float* n_valid, hipStream_t st);
// Per row of logits [rows, ld] (V used columns): loss_rows[r] = lse - logit[target] + z_loss lse^2 (0 when
// the row has no target); with want_grad the logits are overwritten by d(mean loss)/d(logits) =
// (softmax (1 + 2 z_loss lse) - onehot) / max(*n_valid, 1).
hipError_t launch_xent_rows(void* logits, int type, const int32_t* targets, int64_t rows, int V, int ld, float z_loss,
                            const float* n_valid, float* loss_rows, int want_grad, hipStream_t st);
// *loss_out = sum(loss_rows) / max(*n_valid, 1), fixed summation order.
hipError_t launch_loss_reduce(const float* loss_rows, int64_t rows, const float* n_valid, float* loss_out,
                              hipStream_t st);
// out = (accumulate ? out : 0) + alpha * in (float32);  out = alpha * in (storage type)
hipError_t launch_axpy_f32(float* out, const float* in, float alpha, int n, int accumulate, hipStream_t st);
hipError_t launch_scale_vec(void* out, const void* in, float alpha, int n, int type, hipStream_t st);

// ------------------------------------------------------------------ dropout
// out[r * cols + c] = 1 where element (r, c) of the site is kept, 0 where dropped (uint8).
hipError_t launch_dropout_keep(const DropSite& d, int64_t rows, int64_t cols, uint8_t* out, hipStream_t st);
// out[r, c] = in[r, c] * multiplier(r, c) (storage type): the masked, rescaled copy of a gradient that
// feeds the GEMMs of a dropped sublayer output.
hipError_t launch_dropout_apply(const DropSite& d, const void* in, void* out, int type, int64_t rows, int cols,
                                hipStream_t st);

// ------------------------------------------------------------------ measurement aid
// Register-only MFMA loop: each of the 4 waves of a workgroup issues iters * 32 v_mfma_f32_32x32x16_bf16.
hipError_t launch_mfma_peak_probe(int workgroups, int iters, int random_operands, float* sink, hipStream_t st);

// ------------------------------------------------------------------ Adafactor
size_t adafactor_ws_bytes(int64_t rows, int64_t cols, int factored);
hipError_t launch_adafactor(float* param, const float* grad, float* v_row, float* v_col, float* v_full,
                            int64_t rows, int64_t cols, int factored, const adafactor_cfg& c,
                            void* bf16_out, void* ws, hipStream_t st);
// The same update for up to AF_MAX_TENSORS tensors in one sequence of launches.  ws: the tensors'
// workspaces (adafactor_ws_bytes each) back to back, in order.
constexpr int AF_MAX_TENSORS = 16;
struct AfTensor {
  float* param;
  const float* grad;
  float* v_row;
  float* v_col;
  float* v_full;
  int64_t rows, cols;
  int factored;
  void* bf16_out;
  float* m;  // momentum [rows, cols], used when cfg.beta1 > 0
};
hipError_t launch_adafactor_multi(const AfTensor* t, int n, const adafactor_cfg& c, void* ws, hipStream_t st);

}  // namespace t5mi
