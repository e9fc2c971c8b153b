// Ends of the layer stack (paper Sec. 4 models as plain stacks): token-embedding lookup and its
// gradient, and the training loss on the logits -- softmax cross-entropy plus z_loss * log(Z)^2 --
// fused with its gradient.  All of it is bound by HBM bandwidth: the lookup moves 2 T d elements, the
// loss reads every logit once and writes its gradient over it.
#include "kernels.h"

namespace t5mi {

namespace {

// ------------------------------------------------------------------------------------------------
// x[t, :] = E[tok[t], :].  One wave per row, 16-byte accesses when d allows.  Token ids outside
// [0, vocab) are clamped into it (they cannot be rejected on the host: the ids live in device memory).
// ------------------------------------------------------------------------------------------------
template <typename T, int VEC>
__global__ __launch_bounds__(256) void embed_fwd_kernel(const int32_t* __restrict__ tok, const T* __restrict__ E,
                                                        T* __restrict__ x, int64_t rows, int d, int vocab) {
  const int lane = threadIdx.x & 63;
  for (int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); r < rows; r += (int64_t)gridDim.x * 4) {
    int id = tok[r];
    id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
    const T* src = E + (size_t)id * d;
    T* dst = x + (size_t)r * d;
    if constexpr (VEC > 1) {
      typedef __attribute__((ext_vector_type(4))) uint32_t v16;
      constexpr int EPV = 16 / sizeof(T);
      for (int c = lane * EPV; c < d; c += 64 * EPV)
        *reinterpret_cast<v16*>(dst + c) = *reinterpret_cast<const v16*>(src + c);
    } else {
      for (int c = lane; c < d; c += 64) dst[c] = src[c];
    }
  }
}

// dE[tok[t], :] += dx[t, :] in float32 atomics (a token that occurs k times receives k rows).
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_kernel(const int32_t* __restrict__ tok, const T* __restrict__ dx,
                                                        float* __restrict__ dE, int64_t rows, int d, int vocab) {
  const int lane = threadIdx.x & 63;
  for (int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); r < rows; r += (int64_t)gridDim.x * 4) {
    int id = tok[r];
    id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
    float* dst = dE + (size_t)id * d;
    const T* src = dx + (size_t)r * d;
    for (int c = lane; c < d; c += 64) unsafeAtomicAdd(dst + c, to_f32(src[c]));
  }
}

// The same sum in a fixed order: a wave owns kEmbRows consecutive vocabulary rows, scans the token ids 64 at a time
// and, row by row, adds the rows of the positions that hold that id, lowest position first.  No other wave writes
// those rows, so plain read-modify-write is enough and the result does not depend on timing.  The scan costs every
// wave a pass over the ids (from L2) and one compare per owned row and chunk; it is the price of the reproducible
// mode only.
constexpr int kEmbRows = 8;
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_ordered_kernel(const int32_t* __restrict__ tok,
                                                                const T* __restrict__ dx, float* __restrict__ dE,
                                                                int rows, int d, int vocab) {
  const int lane = threadIdx.x & 63;
  const int v0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * kEmbRows;
  if (v0 >= vocab) return;
  for (int r0 = 0; r0 < rows; r0 += 64) {
    const int r = r0 + lane;
    int id = -1;
    if (r < rows) {
      id = tok[r];
      id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
    }
    // (most chunks hold none of this wave's rows: one test for all of them first)
    if (__ballot((unsigned)(id - v0) < (unsigned)kEmbRows) == 0) continue;
#pragma unroll
    for (int q = 0; q < kEmbRows; ++q) {
      unsigned long long hit = __ballot(id == v0 + q);
      while (hit) {
        const int k = __ffsll((long long)hit) - 1;
        hit &= hit - 1;
        float* dst = dE + (size_t)(v0 + q) * d;
        const T* src = dx + (size_t)(r0 + k) * d;
        for (int c = lane; c < d; c += 64) dst[c] += to_f32(src[c]);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Number of positions that carry a loss (0 <= target < vocab), as a float, by one workgroup in a
// fixed order.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void xent_count_kernel(const int32_t* __restrict__ targets, int64_t rows,
                                                          int vocab, float* __restrict__ n_valid) {
  __shared__ int red[16];
  int c = 0;
  for (int64_t r = threadIdx.x; r < rows; r += 1024) c += (targets[r] >= 0 && targets[r] < vocab) ? 1 : 0;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) c += __shfl_xor(c, off, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    int t = 0;
    for (int i = 0; i < 16; ++i) t += red[i];
    *n_valid = (float)t;
  }
}

// loss = sum(loss_rows) / max(n_valid, 1), one workgroup, fixed order (bit-reproducible).
__global__ __launch_bounds__(1024) void loss_reduce_kernel(const float* __restrict__ loss_rows, int64_t rows,
                                                           const float* __restrict__ n_valid,
                                                           float* __restrict__ loss_out) {
  __shared__ float red[16];
  float s = 0.f;
  for (int64_t r = threadIdx.x; r < rows; r += 1024) s += loss_rows[r];
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int i = 0; i < 16; ++i) t += red[i];
    *loss_out = t / fmaxf(*n_valid, 1.f);
  }
}

template <typename T> struct Vec16;
template <> struct Vec16<bf16> { typedef bf16x8 type; };
template <> struct Vec16<float> { typedef f32x4 type; };

template <int NW>
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float m = red[0];
#pragma unroll
  for (int i = 1; i < NW; ++i) m = fmaxf(m, red[i]);
  return m;
}

// Loss row: lse, loss and (GRAD) the gradient written over the logits.
//   lse = m + log sum exp(x - m);  loss = lse - x[target] + z lse^2
//   d loss / d x_v = softmax_v (1 + 2 z lse) - [v == target], times 1 / n_valid
// Rows without a target get loss 0 and a zero gradient.
//
// Register form: one workgroup per row, the whole row is read once with 16-byte loads into NV vectors
// per thread and stays in registers between the reduction and the gradient write.
template <typename T, int NV, bool GRAD>
__global__ __launch_bounds__(256) void xent_rows_vec_kernel(T* __restrict__ logits, const int32_t* __restrict__ targets,
                                                            int V, int ld, float z_loss,
                                                            const float* __restrict__ n_valid,
                                                            float* __restrict__ loss_rows) {
  constexpr int EPV = 16 / sizeof(T);
  typedef __attribute__((ext_vector_type(4))) uint32_t v16;
  typedef typename Vec16<T>::type VT;
  __shared__ float red[4];
  __shared__ float tgt_logit;
  const int64_t row = blockIdx.x;
  T* x = logits + (size_t)row * ld;
  const int tgt = targets[row];
  const bool counted = tgt >= 0 && tgt < V;
  // The row is kept as raw 16-byte vectors; each pass converts on the fly.  The empty asm statements
  // make vector i depend on the result of vector i-1, so that the compiler cannot convert the whole row
  // to float32 first and run all exponentials afterwards (2-4x the registers: one wave per SIMD).
  // Vectors past the end of the row are loaded from its last vector and replaced by -inf, so that the
  // passes below need no per-vector branches (exp(-inf - m) = 0).
  constexpr uint32_t kNegInf = sizeof(T) == 2 ? 0xFF80FF80u : 0xFF800000u;
  v16 raw[NV];
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int c = (i * 256 + threadIdx.x) * EPV;
    const int cc = c < V ? c : V - EPV;
    v16 r = __builtin_nontemporal_load(reinterpret_cast<const v16*>(x + cc));
    if (c >= V) r = v16{kNegInf, kNegInf, kNegInf, kNegInf};
    raw[i] = r;
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const VT v = __builtin_bit_cast(VT, raw[i]);
#pragma unroll
    for (int k = 0; k < EPV; ++k) m = fmaxf(m, to_f32(v[k]));
    __builtin_amdgcn_sched_barrier(0);
  }
  m = block_max<4>(m, red);
  const int rel0 = tgt - (int)threadIdx.x * EPV;
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    asm volatile("" : "+v"(raw[i]), "+v"(s), "+v"(m));  // vector i is not touched before vector i-1 is summed
    const VT v = __builtin_bit_cast(VT, raw[i]);
#pragma unroll
    for (int k = 0; k < EPV; ++k) s += __expf(to_f32(v[k]) - m);
    // one thread owns the target's logit; thread 0 reads it after the barriers of block_sum()
    const int rel = rel0 - i * 256 * EPV;  // position of the target inside this vector, if 0 <= rel < EPV
    if (counted && (unsigned)rel < (unsigned)EPV) {
      float f = 0.f;
#pragma unroll
      for (int k = 0; k < EPV; ++k) f = (rel == k) ? to_f32(v[k]) : f;
      tgt_logit = f;
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  s = block_sum<4>(s, red);
  float lse = m + __logf(s);
  if (threadIdx.x == 0) loss_rows[row] = counted ? lse - tgt_logit + z_loss * lse * lse : 0.f;
  if constexpr (GRAD) {
    // each thread overwrites exactly the vectors it read
    const float inv_n = counted ? 1.f / fmaxf(*n_valid, 1.f) : 0.f;
    const float gain = (1.f + 2.f * z_loss * lse) * inv_n;
    uint32_t chain = 0;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (i * 256 + threadIdx.x) * EPV;
      asm volatile("" : "+v"(raw[i]), "+v"(chain), "+v"(lse));  // one vector at a time, as above
      const int rel = rel0 - i * 256 * EPV;
      const VT v = __builtin_bit_cast(VT, raw[i]);
      VT outv;
#pragma unroll
      for (int k = 0; k < EPV; ++k) {
        float gv = __expf(to_f32(v[k]) - lse) * gain;
        if (rel == k) gv -= inv_n;
        outv[k] = from_f32<T>(gv);
      }
      const v16 ob = __builtin_bit_cast(v16, outv);
      chain = ob[3];
      if (c < V) __builtin_nontemporal_store(ob, reinterpret_cast<v16*>(x + c));
    }
  }
}

// Any V and alignment: the row is read again for each pass (it stays in L2).
template <typename T, bool GRAD>
__global__ __launch_bounds__(256) void xent_rows_generic_kernel(T* __restrict__ logits,
                                                                const int32_t* __restrict__ targets, int V, int ld,
                                                                float z_loss, const float* __restrict__ n_valid,
                                                                float* __restrict__ loss_rows) {
  __shared__ float red[4];
  __shared__ float tgt_logit;
  const int64_t row = blockIdx.x;
  T* x = logits + (size_t)row * ld;
  const int tgt = targets[row];
  const bool counted = tgt >= 0 && tgt < V;
  float m = -INFINITY;
  for (int c = threadIdx.x; c < V; c += 256) m = fmaxf(m, to_f32(x[c]));
  m = block_max<4>(m, red);
  float s = 0.f;
  for (int c = threadIdx.x; c < V; c += 256) {
    const float v = to_f32(x[c]);
    s += __expf(v - m);
    if (c == tgt) tgt_logit = v;  // read by thread 0 after the barriers of block_sum()
  }
  s = block_sum<4>(s, red);
  const float lse = m + __logf(s);
  if (threadIdx.x == 0) loss_rows[row] = counted ? lse - tgt_logit + z_loss * lse * lse : 0.f;
  if constexpr (GRAD) {
    const float inv_n = counted ? 1.f / fmaxf(*n_valid, 1.f) : 0.f;
    const float gain = (1.f + 2.f * z_loss * lse) * inv_n;
    for (int c = threadIdx.x; c < V; c += 256) {
      float gv = __expf(to_f32(x[c]) - lse) * gain;
      if (c == tgt) gv -= inv_n;
      x[c] = from_f32<T>(gv);
    }
  }
}

// out[i] = (accumulate ? out[i] : 0) + alpha * in[i], float32 (scale gradients of the tied-logits form)
__global__ void axpy_f32_kernel(float* __restrict__ out, const float* __restrict__ in, float alpha, int n,
                                int accumulate) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = (accumulate ? out[i] : 0.f) + alpha * in[i];
}
// out[i] = alpha * in[i] in the storage type
template <typename T>
__global__ void scale_vec_kernel(T* __restrict__ out, const T* __restrict__ in, float alpha, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = from_f32<T>(alpha * to_f32(in[i]));
}

__global__ __launch_bounds__(256) void dropout_keep_kernel(DropSite d, int64_t rows, int64_t cols,
                                                            uint8_t* __restrict__ out) {
  const int64_t n = rows * cols;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const uint32_t r = (uint32_t)(i / cols), c = (uint32_t)(i % cols);
    out[i] = drop_mult(d, drop_row_key(d, r), c) != 0.f ? 1 : 0;
  }
}

template <typename T>
// in and out may be the same buffer (a stack drops its end activations in place): no __restrict__.
__global__ __launch_bounds__(256) void dropout_apply_kernel(DropSite d, const T* in, T* out, int64_t rows, int cols) {
  const int lane = threadIdx.x & 63;
  for (int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); r < rows; r += (int64_t)gridDim.x * 4) {
    const uint32_t k1 = drop_row_key(d, (uint32_t)r);
    for (int c = lane; c < cols; c += 64)
      out[r * cols + c] = from_f32<T>(to_f32(in[r * cols + c]) * drop_mult(d, k1, (uint32_t)c));
  }
}

template <typename T, bool GRAD>
hipError_t xent_dispatch(void* logits, const int32_t* targets, int64_t rows, int V, int ld, float z_loss,
                         const float* n_valid, float* loss_rows, hipStream_t st) {
  constexpr int EPV = 16 / sizeof(T);
  const bool vec_ok = V % EPV == 0 && ld % EPV == 0 && ((uintptr_t)logits & 15) == 0;
  const int nv = ceil_div(V, 256 * EPV);
  const dim3 grid((unsigned)rows);
  if (vec_ok && nv <= 4)
    xent_rows_vec_kernel<T, 4, GRAD><<<grid, 256, 0, st>>>((T*)logits, targets, V, ld, z_loss, n_valid, loss_rows);
  else if (vec_ok && nv <= 16)
    xent_rows_vec_kernel<T, 16, GRAD><<<grid, 256, 0, st>>>((T*)logits, targets, V, ld, z_loss, n_valid, loss_rows);
  else
    xent_rows_generic_kernel<T, GRAD><<<grid, 256, 0, st>>>((T*)logits, targets, V, ld, z_loss, n_valid, loss_rows);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_embed_fwd(const int32_t* tokens, const void* E, void* x, int type, int64_t rows, int d, int vocab,
                            hipStream_t st) {
  const int grid = (int)std::min<int64_t>((rows + 3) / 4, 16384);
  const bool vec = (d * (type == IN_BF16 ? 2 : 4)) % 16 == 0 && (((uintptr_t)E | (uintptr_t)x) & 15) == 0;
  if (type == IN_BF16) {
    if (vec) embed_fwd_kernel<bf16, 8><<<grid, 256, 0, st>>>(tokens, (const bf16*)E, (bf16*)x, rows, d, vocab);
    else embed_fwd_kernel<bf16, 1><<<grid, 256, 0, st>>>(tokens, (const bf16*)E, (bf16*)x, rows, d, vocab);
  } else {
    if (vec) embed_fwd_kernel<float, 4><<<grid, 256, 0, st>>>(tokens, (const float*)E, (float*)x, rows, d, vocab);
    else embed_fwd_kernel<float, 1><<<grid, 256, 0, st>>>(tokens, (const float*)E, (float*)x, rows, d, vocab);
  }
  return hipGetLastError();
}

hipError_t launch_embed_bwd(const int32_t* tokens, const void* dx, int type, float* dE, int64_t rows, int d,
                            int vocab, int ordered, hipStream_t st) {
  if (ordered) {
    if (rows > (int64_t)1 << 30) return hipErrorInvalidValue;
    const int grid_v = (vocab + 4 * kEmbRows - 1) / (4 * kEmbRows);
    if (type == IN_BF16)
      embed_bwd_ordered_kernel<bf16><<<grid_v, 256, 0, st>>>(tokens, (const bf16*)dx, dE, (int)rows, d, vocab);
    else
      embed_bwd_ordered_kernel<float><<<grid_v, 256, 0, st>>>(tokens, (const float*)dx, dE, (int)rows, d, vocab);
    return hipGetLastError();
  }
  const int grid = (int)std::min<int64_t>((rows + 3) / 4, 16384);
  if (type == IN_BF16) embed_bwd_kernel<bf16><<<grid, 256, 0, st>>>(tokens, (const bf16*)dx, dE, rows, d, vocab);
  else embed_bwd_kernel<float><<<grid, 256, 0, st>>>(tokens, (const float*)dx, dE, rows, d, vocab);
  return hipGetLastError();
}

hipError_t launch_xent_count(const int32_t* targets, int64_t rows, int vocab, float* n_valid, hipStream_t st) {
  xent_count_kernel<<<1, 1024, 0, st>>>(targets, rows, vocab, n_valid);
  return hipGetLastError();
}

hipError_t launch_xent_rows(void* logits, int type, const int32_t* targets, int64_t rows, int V, int ld, float z_loss,
                            const float* n_valid, float* loss_rows, int want_grad, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  if (type == IN_BF16)
    return want_grad ? xent_dispatch<bf16, true>(logits, targets, rows, V, ld, z_loss, n_valid, loss_rows, st)
                     : xent_dispatch<bf16, false>(logits, targets, rows, V, ld, z_loss, n_valid, loss_rows, st);
  return want_grad ? xent_dispatch<float, true>(logits, targets, rows, V, ld, z_loss, n_valid, loss_rows, st)
                   : xent_dispatch<float, false>(logits, targets, rows, V, ld, z_loss, n_valid, loss_rows, st);
}

hipError_t launch_loss_reduce(const float* loss_rows, int64_t rows, const float* n_valid, float* loss_out,
                              hipStream_t st) {
  loss_reduce_kernel<<<1, 1024, 0, st>>>(loss_rows, rows, n_valid, loss_out);
  return hipGetLastError();
}

hipError_t launch_dropout_keep(const DropSite& d, int64_t rows, int64_t cols, uint8_t* out, hipStream_t st) {
  const int64_t n = rows * cols;
  if (n <= 0) return hipSuccess;
  dropout_keep_kernel<<<(int)std::min<int64_t>((n + 255) / 256, 65536), 256, 0, st>>>(d, rows, cols, out);
  return hipGetLastError();
}

hipError_t launch_dropout_apply(const DropSite& d, const void* in, void* out, int type, int64_t rows, int cols,
                                hipStream_t st) {
  const int grid = (int)std::min<int64_t>((rows + 3) / 4, 16384);
  if (type == IN_BF16)
    dropout_apply_kernel<bf16><<<grid, 256, 0, st>>>(d, (const bf16*)in, (bf16*)out, rows, cols);
  else
    dropout_apply_kernel<float><<<grid, 256, 0, st>>>(d, (const float*)in, (float*)out, rows, cols);
  return hipGetLastError();
}

hipError_t launch_axpy_f32(float* out, const float* in, float alpha, int n, int accumulate, hipStream_t st) {
  axpy_f32_kernel<<<ceil_div(n, 256), 256, 0, st>>>(out, in, alpha, n, accumulate);
  return hipGetLastError();
}

hipError_t launch_scale_vec(void* out, const void* in, float alpha, int n, int type, hipStream_t st) {
  if (type == IN_BF16) scale_vec_kernel<bf16><<<ceil_div(n, 256), 256, 0, st>>>((bf16*)out, (const bf16*)in, alpha, n);
  else scale_vec_kernel<float><<<ceil_div(n, 256), 256, 0, st>>>((float*)out, (const float*)in, alpha, n);
  return hipGetLastError();
}

}  // namespace t5mi
