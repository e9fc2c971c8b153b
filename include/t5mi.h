/*
 * t5mi.h - C ABI of the MI355X (gfx950) implementation of one T5.1.1-style
 * Transformer block (encoder layer, decoder-only layer, or encoder-decoder
 * decoder layer with cross-attention): forward, backward, relative-position
 * buckets and the Adafactor update of its weights; of whole stacks of such
 * layers with embedding, final norm, logits and loss (one stack, or the
 * encoder-decoder pair); and of the dropout mask generator they share.
 *
 * The paper (Sec. 4, "Example models") ships T5.1.1 and a decoder-only model as
 * its reference architectures and Sec. 2.3 describes them as ordinary layer
 * stacks; the block below is one layer of those stacks.  The paper prints no
 * layer formulas, so each entry point states the public definition it computes.
 *
 * Conventions for every call
 *   - returns an int status (T5_OK == 0); never throws, aborts or prints;
 *   - all tensor pointers are DEVICE pointers owned by the caller, dense
 *     row-major, no strides, no aliasing between inputs and outputs;
 *   - config structs are HOST pointers, read during the call only;
 *   - the library allocates no device memory: scratch comes from the caller's
 *     workspace, whose size is returned by the *_bytes() queries (0 on an
 *     invalid config).  Host-side objects only: the stack entry points build
 *     short host arrays per call, and the two opt-in aids create HIP objects
 *     (t5_wgrad_overlap_enable: one stream and two events, kept until it is
 *     switched off; t5_step_timing_enable: one event pair per timed step);
 *   - one host thread at a time: the opt-in aids and the one-time kernel
 *     attribute set-up keep process-wide state without locks;
 *   - all device work is enqueued on `stream` (a hipStream_t passed as void*;
 *     NULL = the default stream) and the call returns without synchronising
 *     (after t5_wgrad_overlap_enable(1) the backward passes also use one stream
 *     of the library's own, ordered against `stream` with events);
 *   - arguments are validated before the first HIP call, so error paths can be
 *     exercised on a host without a GPU.
 */
#ifndef T5MI_H
#define T5MI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  T5_OK = 0,
  T5_ERR_NULL = 1,        /* a required pointer is NULL */
  T5_ERR_SHAPE = 2,       /* non-positive or inconsistent dimension / hyper-parameter */
  T5_ERR_UNSUPPORTED = 3, /* valid problem, but no kernel for this shape/dtype */
  T5_ERR_WORKSPACE = 4,   /* workspace_bytes smaller than the query result */
  T5_ERR_DEVICE = 5       /* a HIP call or kernel launch failed */
};

enum { T5_F32 = 0, T5_BF16 = 1 };

/* Feed-forward sublayer of a block (paper Sec. 4 names both T5 generations):
 *   T5_MLP_GEGLU_TANH  T5.1.1: (gelu_tanh(n2 Wi0) * (n2 Wi1)) Wo_ff
 *   T5_MLP_RELU        original T5: max(n2 Wi0, 0) Wo_ff; wi1 and its gradient pointer are ignored
 *   T5_MLP_GEGLU_ERF   the gated form with the exact GELU z Phi(z) */
enum { T5_MLP_GEGLU_TANH = 0, T5_MLP_RELU = 1, T5_MLP_GEGLU_ERF = 2 };

/* One Transformer block (paper Sec. 4: T5.1.1 encoder layer, or a decoder-only layer when
 * causal != 0):
 *   n1 = RMSNorm(x; ln1_scale)                      r = (mean_c x_c^2 + rms_eps)^-1/2, no mean subtraction
 *   q,k,v = n1 Wq, n1 Wk, n1 Wv                     column h*d_kv + c = head h, channel c; no biases
 *   s[h,i,j] = attn_scale <q_hi,k_hj> + rel_table[bucket(j-i), h];   causal: j > i masked
 *   h = x + concat_h(softmax_j(s) v) Wo
 *   n2 = RMSNorm(h; ln2_scale);  y = h + (gelu_tanh(n2 Wi0) * (n2 Wi1)) Wo_ff
 * bucket() is t5_relpos_bucket() with bidirectional = !causal. */
typedef struct {
  int32_t batch, seq, d_model, n_heads, d_kv, d_ff;
  int32_t num_buckets;  /* 32 in T5 */
  int32_t max_distance; /* 128 in T5 */
  int32_t causal;       /* 0: bidirectional buckets, no mask; 1: unidirectional buckets + causal mask */
  int32_t dtype;        /* T5_F32 or T5_BF16: storage type of x, y, dy, dx and all weights */
  float rms_eps;        /* 1e-6 in T5 */
  float attn_scale;     /* 1.0 = T5 convention (scale folded into the initialisation) */
  int32_t mlp_kind;     /* T5_MLP_*; 0 = the T5.1.1 gated tanh-GELU */
  float dropout_rate;   /* 0 = none (pre-training of T5.1.1); in (0, 1): training-time dropout, see t5_dropout_keep */
  uint32_t dropout_seed_lo, dropout_seed_hi; /* 64-bit seed; a caller changes it per step and per layer */
  int32_t deterministic; /* 0: the partial sums of the weight gradients (reduction over all tokens, split across
                            workgroups) and of the bias-table gradient meet in float32 atomics: results are
                            reproducible to float32 rounding.  1: they are written out and added in a fixed order
                            by a second pass: every output of the backward pass is bit-reproducible, for a larger
                            workspace (the *_workspace_bytes() queries account for it) and a few percent of time.
                            Applies to the matrix-unit kernels; y, dx (and denc) are bit-reproducible either way.
                            In a stack it also covers the output-matrix gradient and the embedding gradient (formed
                            per vocabulary row in position order instead of with atomics). */
} t5_block_cfg;

/* Weights, device pointers, element type cfg.dtype, row-major [in, out]. */
typedef struct {
  const void* ln1_scale; /* [d_model] */
  const void* wq;        /* [d_model, n_heads*d_kv] */
  const void* wk;        /* [d_model, n_heads*d_kv] */
  const void* wv;        /* [d_model, n_heads*d_kv] */
  const void* wo;        /* [n_heads*d_kv, d_model] */
  const void* rel_table; /* [num_buckets, n_heads] */
  const void* ln2_scale; /* [d_model] */
  const void* wi0;       /* [d_model, d_ff]; this branch goes through GELU */
  const void* wi1;       /* [d_model, d_ff]; linear gate */
  const void* wo_ff;     /* [d_ff, d_model] */
} t5_block_weights;

/* Weight gradients, device pointers, always float32, same shapes as the weights. */
typedef struct {
  float* ln1_scale;
  float* wq;
  float* wk;
  float* wv;
  float* wo;
  float* rel_table;
  float* ln2_scale;
  float* wi0;
  float* wi1;
  float* wo_ff;
} t5_block_grads;

/* Relative-position bucket of T5 (used by the models of paper Sec. 4), elementwise:
 * rel_pos = key_position - query_position.  Half of the buckets (per sign when bidirectional)
 * are exact offsets, the rest are logarithmically spaced up to max_distance; the boundaries are
 * evaluated in exact integer arithmetic.  rel_pos, bucket: device int32[n].  n == 0 is a no-op.
 * Errors: NULL pointer with n > 0 -> T5_ERR_NULL; n < 0, num_buckets < 2 (or odd / < 4 when
 * bidirectional), max_distance <= exact range -> T5_ERR_SHAPE; more than 64 logarithmic
 * buckets per side -> T5_ERR_UNSUPPORTED. */
int t5_relpos_bucket(const int32_t* rel_pos, int32_t* bucket, int64_t n, int bidirectional,
                     int num_buckets, int max_distance, void* stream);

/* Dropout of the T5 models (paper Sec. 4; used when fine-tuning) at the block's four sites: attention
 * probabilities (site 1; row = (batch*n_heads + head)*seq + query, column = key), output of the attention
 * sublayer before the residual add (site 2; row = token, column = channel), feed-forward hidden
 * activation (site 3; column = hidden unit) and output of the feed-forward sublayer (site 4).  Kept
 * elements are multiplied by 1/(1 - rate).  The generator is counter-based and stateless: with
 * mix32(x): x ^= x>>16; x *= 0x7FEB352D; x ^= x>>15; x *= 0x846CA68B; x ^= x>>16 (mod 2^32),
 *   keep(row, col) = mix32(mix32(k0 ^ row ^ seed_hi) ^ col) >= floor(rate * 2^32),
 *   k0 = mix32(seed_lo ^ site * 0x9E3779B9),
 * so the forward and backward kernels regenerate the same mask from (seed, site, row, col) and nothing is
 * stored.  t5_dropout_keep writes that mask (1 = kept) for inspection and tests: keep is device
 * uint8 [rows, cols].  Errors: NULL -> T5_ERR_NULL; rows/cols < 0, rate outside [0, 1) -> T5_ERR_SHAPE.
 * Every entry point applies it when its block configuration has dropout_rate > 0.  The decoder layer adds
 * site 5 (cross-attention probabilities; row = (batch*n_heads + head)*seq + query, column = encoder
 * position) and site 6 (output of the cross-attention sublayer).  A stack runs layer l (0-based) with the
 * seed  seed + (l + 1) * 0x9E3779B97F4A7C15 (mod 2^64)  and applies site 7 to the embedded tokens and site
 * 8 to the output of the final norm, both under the configuration's own seed; in the encoder-decoder pair
 * each side takes rate and seed from its block configuration, the decoder's layers count on from the
 * encoder's (l = n_enc_layers + index), and the decoder's ends are sites 9 and 10. */
int t5_dropout_keep(uint64_t seed, int site, float rate, int64_t rows, int64_t cols, uint8_t* keep,
                    void* stream);

/* Bytes of the saved-for-backward buffer written by t5_block_fwd and read by t5_block_bwd
 * (opaque layout), and of the scratch workspace (max over forward and backward). */
size_t t5_block_stash_bytes(const t5_block_cfg* cfg);
size_t t5_block_workspace_bytes(const t5_block_cfg* cfg);

/* Which kernels a configuration runs on (a pure host-side query: no device work, usable without a GPU).
 * Returns a bit mask, or -1 for an invalid configuration.  enc_seq = 0: the block; > 0: the decoder layer
 * with cross-attention over enc_seq positions.  A clear bit means the general-shape kernels (any shape,
 * reference-grade speed) take that part; results obey the same bounds either way. */
enum {
  T5_PATH_MFMA_GEMM = 1,       /* forward projections on the matrix-unit GEMM, gated activation fused into it */
  T5_PATH_MFMA_ATTN_FWD = 2,   /* fused matrix-unit self-attention, forward */
  T5_PATH_MFMA_ATTN_BWD = 4,   /* ... backward */
  T5_PATH_MFMA_CROSS_ATTN = 8  /* fused matrix-unit cross-attention (decoder layer), both directions */
};
int t5_block_kernel_path(const t5_block_cfg* cfg, int32_t enc_seq);

/* Forward of the block defined at t5_block_cfg.  x, y: [batch, seq, d_model] of cfg.dtype.
 * stash: t5_block_stash_bytes(cfg) bytes, 256-byte aligned, written here.
 * Errors: NULL -> T5_ERR_NULL; bad dims -> T5_ERR_SHAPE; shape without a kernel ->
 * T5_ERR_UNSUPPORTED; small workspace -> T5_ERR_WORKSPACE; launch failure -> T5_ERR_DEVICE. */
int t5_block_fwd(const t5_block_cfg* cfg, const void* x, const t5_block_weights* w, void* y,
                 void* stash, void* workspace, size_t workspace_bytes, void* stream);

/* Backward of the same block: given dy = dL/dy, writes dx = dL/dx (cfg.dtype) and the float32
 * weight gradients (all ten pointers required).  accumulate == 0 overwrites the gradients,
 * accumulate != 0 adds to them.  x, w and stash must be those of the matching forward call. */
int t5_block_bwd(const t5_block_cfg* cfg, const void* dy, const void* x, const t5_block_weights* w,
                 const void* stash, void* dx, const t5_block_grads* dw, int accumulate,
                 void* workspace, size_t workspace_bytes, void* stream);

/* Decoder layer of the encoder-decoder T5.1.1 (paper Sec. 4): the block above with a
 * cross-attention sublayer between self-attention and the MLP.  With h1 the residual stream after
 * self-attention (cfg.causal selects the decoder's causal mask and unidirectional buckets) and
 * enc [batch, enc_seq, d_model] the encoder stack's output:
 *   nx = RMSNorm(h1; lnx_scale);  q = nx Xq;  k = enc Xk;  v = enc Xv        (heads as above)
 *   s[h,i,j] = attn_scale <q_hi,k_hj>     no position bias, no mask, i < seq, j < enc_seq
 *   h2 = h1 + concat_h(softmax_j(s) v) Xo;   then n2 = RMSNorm(h2; ln2_scale), y = h2 + MLP(n2).
 * Cross-attention weights and gradients; the rest of the layer uses t5_block_weights / _grads. */
typedef struct {
  const void* lnx_scale; /* [d_model] */
  const void* xq;        /* [d_model, n_heads*d_kv] */
  const void* xk;        /* [d_model, n_heads*d_kv] */
  const void* xv;        /* [d_model, n_heads*d_kv] */
  const void* xo;        /* [n_heads*d_kv, d_model] */
} t5_cross_weights;
typedef struct {
  float* lnx_scale;
  float* xq;
  float* xk;
  float* xv;
  float* xo;
} t5_cross_grads;

/* Stash / workspace sizes of the decoder layer (0 on an invalid config or enc_seq < 1). */
size_t t5_decoder_block_stash_bytes(const t5_block_cfg* cfg, int32_t enc_seq);
size_t t5_decoder_block_workspace_bytes(const t5_block_cfg* cfg, int32_t enc_seq);

/* Forward of the decoder layer.  x, y: [batch, seq, d_model]; enc: [batch, enc_seq, d_model]; all of
 * cfg.dtype.  stash: t5_decoder_block_stash_bytes() bytes, 256-byte aligned, written here.
 * Errors as t5_block_fwd; enc_seq < 1 -> T5_ERR_SHAPE. */
int t5_decoder_block_fwd(const t5_block_cfg* cfg, int32_t enc_seq, const void* x, const void* enc,
                         const t5_block_weights* w, const t5_cross_weights* xw, void* y, void* stash,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Backward of the decoder layer: writes dx [batch, seq, d_model] and denc [batch, enc_seq, d_model]
 * (cfg.dtype; denc is overwritten, a caller with several decoder layers sums them) and the float32
 * weight gradients of both structs (all fifteen pointers required; accumulate as in t5_block_bwd).
 * x, enc, w, xw and stash must be those of the matching forward call. */
int t5_decoder_block_bwd(const t5_block_cfg* cfg, int32_t enc_seq, const void* dy, const void* x,
                         const void* enc, const t5_block_weights* w, const t5_cross_weights* xw,
                         const void* stash, void* dx, void* denc, const t5_block_grads* dw,
                         const t5_cross_grads* dxw, int accumulate, void* workspace,
                         size_t workspace_bytes, void* stream);

/* A stack of n_layers identical blocks with its two ends (paper Sec. 4: the decoder-only model when
 * block.causal != 0, an encoder-style stack otherwise; Sec. 2.3: models are plain layer stacks):
 *   x_0 = E[tokens]                               token embedding, no input scaling
 *   x_{l+1} = block_l(x_l)                        the block above; ONE relative-position table serves
 *                                                 every layer (its gradient is the sum over layers)
 *   nf = RMSNorm(x_L; final_scale)
 *   logits = nf Wout                              tied_logits != 0: logits = d_model^-1/2 nf E^T
 *   loss = mean over positions with 0 <= target < vocab of
 *          lse - logits[target] + z_loss lse^2,   lse = log sum_v exp(logits_v)
 * remat == 0 keeps every layer's saved activations between the forward and the backward sweep, and
 * (bf16 stacks without dropout) every layer's backward workspace until the sweep is over, so that the
 * weight gradients of all layers are computed by one grouped GEMM per kind of weight afterwards;
 * remat != 0 keeps the layer inputs only and recomputes each layer's forward inside the backward
 * sweep (one extra forward per layer and per-layer weight-gradient GEMMs, for a fraction of the
 * memory: t5_stack_workspace_bytes() tells). */
typedef struct {
  t5_block_cfg block; /* per-layer shapes; block.batch x block.seq tokens per step */
  int32_t n_layers;
  int32_t vocab;
  int32_t tied_logits;
  int32_t remat;
  float z_loss; /* 1e-4 in the T5 recipe; 0 gives plain cross-entropy */
} t5_stack_cfg;

/* Device pointers of cfg.block.dtype.  layers: HOST array of n_layers structs of device pointers;
 * their rel_table fields are ignored (the stack's shared table is used). */
typedef struct {
  const void* embedding;          /* [vocab, d_model] */
  const void* rel_table;          /* [num_buckets, n_heads], shared by all layers */
  const t5_block_weights* layers; /* [n_layers] */
  const void* final_scale;        /* [d_model] */
  const void* logits_w;           /* [d_model, vocab]; ignored when tied_logits */
} t5_stack_weights;

/* float32 gradients, same shapes.  layers[l].rel_table is ignored. */
typedef struct {
  float* embedding;
  float* rel_table;
  const t5_block_grads* layers; /* HOST array [n_layers] */
  float* final_scale;
  float* logits_w; /* ignored when tied_logits */
} t5_stack_grads;

/* Bytes of workspace for t5_stack_loss_and_grad (activations of all layers, or of one with remat,
 * the logits of one chunk of tokens, scratch).  0 on an invalid config. */
size_t t5_stack_workspace_bytes(const t5_stack_cfg* cfg);

/* One training step's forward and backward: writes the loss (one float32, device memory) and, unless
 * grads == NULL (then only the loss is computed), every gradient.  tokens, targets: device int32
 * [batch, seq]; token ids are clamped into [0, vocab); targets outside [0, vocab) carry no loss (use -1
 * for padding).  accumulate as in t5_block_bwd.  The logits are produced and consumed a chunk of
 * tokens at a time (logits GEMM, loss and its gradient over the logits in place, the two gradient
 * GEMMs), so the [tokens, vocab] matrix never exists in full.
 * Errors: as t5_block_fwd; n_layers < 1, vocab < 2, z_loss < 0 or not finite -> T5_ERR_SHAPE. */
int t5_stack_loss_and_grad(const t5_stack_cfg* cfg, const int32_t* tokens, const int32_t* targets,
                           const t5_stack_weights* w, float* loss, const t5_stack_grads* grads,
                           int accumulate, void* workspace, size_t workspace_bytes, void* stream);

/* The encoder-decoder model (paper Sec. 4: T5.1.1): an encoder stack of bidirectional blocks and a
 * decoder stack of causal blocks with cross-attention (t5_decoder_block_*), sharing one token
 * embedding:
 *   enc_out = RMSNorm(encoder_layers(E[enc_tokens]); enc_final_scale)
 *   x_{l+1} = decoder_block_l(x_l, enc_out),  x_0 = E[dec_tokens]
 *   nf = RMSNorm(x_L; dec_final_scale);  logits and loss as for t5_stack_cfg
 * Each stack has its own shared relative-position table (bidirectional / unidirectional buckets);
 * cross-attention has none.  The gradient of enc_out is the sum over the decoder layers.
 * enc_block.causal must be 0, dec_block.causal != 0; batch, d_model and dtype must agree;
 * enc_block.seq is the encoder length, dec_block.seq the decoder length. */
typedef struct {
  t5_block_cfg enc_block;
  t5_block_cfg dec_block;
  int32_t n_enc_layers, n_dec_layers;
  int32_t vocab;
  int32_t tied_logits;
  int32_t remat;
  float z_loss;
} t5_encdec_cfg;

typedef struct {
  const void* embedding;              /* [vocab, d_model], shared by encoder and decoder */
  const void* enc_rel_table;          /* [num_buckets, n_heads] */
  const t5_block_weights* enc_layers; /* HOST array [n_enc_layers]; rel_table fields ignored */
  const void* enc_final_scale;        /* [d_model] */
  const void* dec_rel_table;
  const t5_block_weights* dec_layers; /* HOST array [n_dec_layers] */
  const t5_cross_weights* dec_cross;  /* HOST array [n_dec_layers] */
  const void* dec_final_scale;
  const void* logits_w;               /* [d_model, vocab]; ignored when tied_logits */
} t5_encdec_weights;

typedef struct {
  float* embedding;
  float* enc_rel_table;
  const t5_block_grads* enc_layers;
  float* enc_final_scale;
  float* dec_rel_table;
  const t5_block_grads* dec_layers;
  const t5_cross_grads* dec_cross;
  float* dec_final_scale;
  float* logits_w;
} t5_encdec_grads;

size_t t5_encdec_workspace_bytes(const t5_encdec_cfg* cfg);

/* Loss and gradients of the encoder-decoder model; arguments as t5_stack_loss_and_grad, with
 * enc_tokens [batch, enc_block.seq] and dec_tokens, targets [batch, dec_block.seq].
 * Errors: as t5_stack_loss_and_grad; mismatched encoder / decoder configs -> T5_ERR_SHAPE. */
int t5_encdec_loss_and_grad(const t5_encdec_cfg* cfg, const int32_t* enc_tokens, const int32_t* dec_tokens,
                            const int32_t* targets, const t5_encdec_weights* w, float* loss,
                            const t5_encdec_grads* grads, int accumulate, void* workspace,
                            size_t workspace_bytes, void* stream);

/* Adafactor (the optimizer of the T5 models of paper Sec. 4) with factored second moments and
 * update clipping, no momentum, no weight decay, for one [rows, cols] float32 tensor:
 *   beta2 = 1 - step^-decay_pow;  Q = G*G + eps1
 *   factored:  v_row <- beta2 v_row + (1-beta2) mean_j Q;  v_col likewise over rows;
 *              vhat_ij = v_row_i v_col_j / mean_i v_row_i
 *   otherwise: v_full <- beta2 v_full + (1-beta2) Q;  vhat = v_full
 *   U = G / sqrt(vhat);  U <- U / max(1, RMS(U)/clip)
 *   D = lr * (scale_by_param ? max(eps2, RMS(param)) : 1) * U
 *   beta1 > 0 (adafactor_step_multi only):  m <- beta1 m + (1 - beta1) D;  D = m        (momentum)
 *   param <- param - D - lr * weight_decay * param                                       (decoupled decay)
 * beta1 = 0 and weight_decay = 0 give the plain update.  param and the state are updated in place.  bf16_copy_out (nullable) receives the new
 * parameters rounded to bf16.  Unused state pointers may be NULL.
 * Errors: NULL -> T5_ERR_NULL; rows/cols < 1, step < 1, clip <= 0, beta1 outside [0, 1),
 * weight_decay < 0 -> T5_ERR_SHAPE; small workspace -> T5_ERR_WORKSPACE; beta1 > 0 through
 * adafactor_step (which has no momentum buffer) -> T5_ERR_UNSUPPORTED. */
typedef struct {
  float lr;
  float decay_pow; /* 0.8 */
  float eps1;      /* 1e-30 */
  float eps2;      /* 1e-3 */
  float clip;      /* 1.0 */
  int32_t scale_by_param;
  int32_t step; /* 1-based */
  float beta1;        /* 0: no momentum; else in (0, 1) and every tensor needs its m buffer */
  float weight_decay; /* 0: none; >= 0 */
} adafactor_cfg;

size_t adafactor_workspace_bytes(int64_t rows, int64_t cols, int factored);
int adafactor_step(float* param, const float* grad, float* v_row, float* v_col, float* v_full,
                   int64_t rows, int64_t cols, int factored, const adafactor_cfg* cfg,
                   void* bf16_copy_out, void* workspace, size_t workspace_bytes, void* stream);

/* adafactor_step for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving or training loops, harnesses that forbid allocation.  Same arguments, results and
 * errors as adafactor_step, without workspace / workspace_bytes: the scratch is a fixed device array of
 * ADAFACTOR_STATIC_SCRATCH_BYTES inside the library (each GPU the library runs on holds its own copy until
 * the process ends).  A tensor whose adafactor_workspace_bytes() exceeds that size is refused with
 * T5_ERR_WORKSPACE before any device work.  The call allocates nothing and frees nothing.  All calls on one GPU
 * share that GPU's array: calls that may overlap on one GPU (different streams, different host threads) race
 * and must be serialised by the caller; calls in stream order on one stream are safe. */
#define ADAFACTOR_STATIC_SCRATCH_BYTES (4u << 20)
int adafactor_step_static(float* param, const float* grad, float* v_row, float* v_col, float* v_full,
                          int64_t rows, int64_t cols, int factored, const adafactor_cfg* cfg,
                          void* bf16_copy_out, void* stream);

/* The same update for several tensors at once (the ten parameter tensors of a block): one sequence
 * of five launches for the whole set instead of five per tensor, which is what the step costs at
 * T5.1.1-Small/Base sizes.  Each entry is what adafactor_step takes for one tensor; every tensor
 * gets the same cfg (paper Sec. 4 trains all parameters with one optimizer setting).  workspace: at
 * least adafactor_multi_workspace_bytes() (the per-tensor workspaces back to back).  Results are
 * identical to calling adafactor_step per tensor.  Longer lists (all tensors of a stack) are processed
 * 16 consecutive entries at a time, in stream order, the groups sharing the workspace:
 * adafactor_multi_workspace_bytes() is the largest group's need.
 * Errors: as adafactor_step; n_tensors < 1 -> T5_ERR_SHAPE, > 65536 -> T5_ERR_UNSUPPORTED. */
typedef struct {
  float* param;
  const float* grad;
  float* v_row;  /* [rows] if factored */
  float* v_col;  /* [cols] if factored */
  float* v_full; /* [rows, cols] if not factored */
  int64_t rows, cols;
  int32_t factored;
  void* bf16_copy_out; /* nullable */
  float* m;            /* [rows, cols] momentum, required when cfg.beta1 > 0, else ignored */
} adafactor_tensor;
size_t adafactor_multi_workspace_bytes(const adafactor_tensor* tensors, int n_tensors);
int adafactor_step_multi(const adafactor_tensor* tensors, int n_tensors, const adafactor_cfg* cfg,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Building block of the block's projections (paper Sec. 4 models are stacks of such matmuls):
 * C[m,n] = sum_k A(m,k) B(n,k), bf16 operands, float32 accumulation on the MFMA units, float32 C
 * [M, ldc].  a_kc != 0: A(m,k) = A[m*lda + k], else A[k*lda + m]; b_kc likewise for B(n,k).
 * Only a_kc == b_kc is implemented.  Exposed for unit tests and per-kernel timing.
 * Errors: NULL -> T5_ERR_NULL; M,N,K < 1 -> T5_ERR_SHAPE; K % 64, lda/ldb % 8, pointers not
 * 16-byte aligned, (m-contiguous case) M or N % 8 -> T5_ERR_UNSUPPORTED. */
int t5_gemm_bf16(const void* A, const void* B, float* C, int M, int N, int K, int lda, int ldb, int ldc,
                 int a_kc, int b_kc, void* stream);

/* Opt-in overlap inside the backward passes.  The weight-gradient GEMMs are leaves of the backward's
 * dependency graph; after t5_wgrad_overlap_enable(1) every backward entry point launches them on a
 * second stream owned by the library (default priority, created by that call, ordered against the caller's
 * stream with events: forked after the producers of each GEMM's operands, joined before the call returns
 * or the next layer starts), so that they run beside the chain that carries the gradient to the input.
 * Results are identical up to the order of the float32 atomic additions.  The state is per process and
 * not thread-safe; call it outside stream capture.  Passes with dropout, and passes on a stream that is
 * being captured into a graph, stay on one stream.  t5_wgrad_overlap_enable(0) drains and releases the stream.
 * Returns T5_OK or T5_ERR_DEVICE. */
int t5_wgrad_overlap_enable(int enable);

/* Per-step device timing of t5_block_fwd / t5_block_bwd for roofline reports.  While enabled, every
 * step of the block is bracketed by HIP events on the caller's stream; t5_step_timing_read()
 * synchronises those events and returns, per step, the summed milliseconds and the number of
 * launches since the last t5_step_timing_enable(1).  names/ms/calls hold up to `cap` entries; the
 * return value is the number of steps recorded.  Name pointers stay valid for the process. */
void t5_step_timing_enable(int enable);
int t5_step_timing_read(const char** names, float* ms, int* calls, int cap);

/* Measurement aid for the roofline report: `workgroups` workgroups of 4 waves each issue
 * iters * 32 v_mfma_f32_32x32x16_bf16 per wave on register operands (no LDS, no memory traffic):
 * 2 * 32*32*16 FLOP per instruction.  random_operands != 0 fills the operands with pseudo-random
 * bf16 values instead of ones: the rate then shows the clock the part sustains under the switching
 * activity of real data.  sink: device buffer of >= 256 floats (practically never written).  The
 * caller times it.  Errors: sizes < 1 -> T5_ERR_SHAPE, NULL -> T5_ERR_NULL. */
int t5_mfma_peak_probe(int workgroups, int iters, int random_operands, float* sink, void* stream);

const char* t5_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* T5MI_H */
