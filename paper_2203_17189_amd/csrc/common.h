// Internal helpers shared by the HIP kernels of the T5 block library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/t5mi.h"

namespace t5mi {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kWave = 64;

// ---- storage-type conversion (round to nearest even for bf16) ----
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  bf16x2 p;
  p[0] = (bf16)lo;
  p[1] = (bf16)hi;
  return __builtin_bit_cast(uint32_t, p);
}

// ---- wavefront (64 lanes) and workgroup reductions ----
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
// Sum over a workgroup of NW waves; every thread gets the result.  `red` holds >= NW floats of LDS.
template <int NW>
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  if (NW == 1) return v;
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NW; ++i) s += red[i];
  return s;
}

// tanh-form GELU, float32.  0.5 (1 + tanh(y)) = 1 / (1 + e^(-2y)), so
//   gelu(z) = z * s,  s = sigmoid(2 kappa (z + beta z^3)),
//   gelu'(z) = s + z s (1 - s) * 2 kappa (1 + 3 beta z^2),
// with one exp2 and one reciprocal (absolute error ~1e-7).  Saturates without NaNs: s -> 0 for
// large negative z (exp2 -> inf, rcp -> 0), s -> 1 for large positive z.
__device__ __forceinline__ float gelu_gate(float z, float z2) {
  constexpr float c = -2.f * 0.7978845608028654f * 1.4426950408889634f;  // -2 kappa log2(e), folded into the cubic
  return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(z * fmaf(z2, c * 0.044715f, c)));
}
__device__ __forceinline__ float gelu_tanh(float z) { return z * gelu_gate(z, z * z); }
__device__ __forceinline__ void gelu_tanh_both(float z, float& g, float& dg) {
  constexpr float k2 = 2.f * 0.7978845608028654f;
  const float z2 = z * z;
  const float s = gelu_gate(z, z2);
  g = z * s;
  // g (1 - s) = g - g s, and 2 kappa (1 + 3 beta z^2) as one fma
  dg = fmaf(fmaf(-g, s, g), fmaf(z2, k2 * 3.f * 0.044715f, k2), s);
}

// Exact GELU z Phi(z) and its derivative Phi(z) + z phi(z).
__device__ __forceinline__ void gelu_erf_both(float z, float& g, float& dg) {
  const float cdf = 0.5f * (1.f + erff(z * 0.7071067811865476f));
  g = z * cdf;
  dg = fmaf(z * 0.3989422804014327f, __expf(-0.5f * z * z), cdf);
}
enum { ACT_GELU_TANH = 0, ACT_RELU = 1, ACT_GELU_ERF = 2 };
__device__ __forceinline__ void gelu_both(int act, float z, float& g, float& dg) {
  if (act == ACT_GELU_ERF) gelu_erf_both(z, g, dg);
  else gelu_tanh_both(z, g, dg);
}

// ---- dropout with a counter-based generator ----
// A 32-bit finaliser (xor-shift / odd-multiply rounds with the public-domain "lowbias32" constants); a
// bijection on 32 bits.  Element (hi, lo) of a dropout site is kept iff
//   mix32(mix32(k0 ^ hi ^ seed_hi) ^ lo) >= floor(rate * 2^32),   k0 = mix32(seed_lo ^ site * 0x9E3779B9),
// a pure function of (seed, site, hi, lo): the forward, the backward and any tiling regenerate it.
__host__ __device__ inline uint32_t mix32(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7FEB352Du;
  x ^= x >> 15;
  x *= 0x846CA68Bu;
  x ^= x >> 16;
  return x;
}
struct DropSite {
  uint32_t k0, seed_hi, thr;
  float scale;  // 1 / (1 - rate)
  int on;       // rate > 0
};
inline DropSite make_drop_site(uint64_t seed, int site, float rate) {
  DropSite d;
  d.on = rate > 0.f ? 1 : 0;
  d.k0 = mix32((uint32_t)seed ^ ((uint32_t)site * 0x9E3779B9u));
  d.seed_hi = (uint32_t)(seed >> 32);
  const double t = (double)(rate > 0.f ? rate : 0.f) * 4294967296.0;
  d.thr = t >= 4294967295.0 ? 0xFFFFFFFFu : (uint32_t)t;
  d.scale = 1.f / (1.f - (rate > 0.f ? rate : 0.f));
  return d;
}
// Sites: the block's four; the cross-attention sublayer of a decoder layer (probabilities, output); the ends
// of a stack (embedded tokens, output of the final norm), with their own numbers on the decoder side of an
// encoder-decoder pair.
enum {
  DROP_ATTN_PROBS = 1, DROP_ATTN_OUT = 2, DROP_MLP_HIDDEN = 3, DROP_MLP_OUT = 4, DROP_CROSS_PROBS = 5,
  DROP_CROSS_OUT = 6, DROP_EMBED = 7, DROP_FINAL = 8, DROP_DEC_EMBED = 9, DROP_DEC_FINAL = 10
};
__device__ __forceinline__ uint32_t drop_row_key(const DropSite& d, uint32_t hi) { return mix32(d.k0 ^ hi ^ d.seed_hi); }
// multiplier of element lo in the row whose key is k1: scale where kept, 0 where dropped
__device__ __forceinline__ float drop_mult(const DropSite& d, uint32_t k1, uint32_t lo) {
  return mix32(k1 ^ lo) >= d.thr ? d.scale : 0.f;
}

// Threshold table of the logarithmic relative-position buckets, built on the host in exact
// integer arithmetic and passed to kernels by value.
struct RelposLut {
  int32_t bidirectional;
  int32_t n_side;     // buckets per side
  int32_t max_exact;  // offsets below this are their own bucket
  int32_t n_thr;      // number of thresholds in thr[]
  int32_t thr[64];    // thr[m] = smallest distance whose logarithmic index is >= m+1
};

__device__ __forceinline__ int relpos_bucket_dev(int rp, const RelposLut& lut) {
  int base = 0, n;
  if (lut.bidirectional) {
    if (rp > 0) base = lut.n_side;
    n = rp < 0 ? -rp : rp;
  } else {
    n = rp < 0 ? -rp : 0;
  }
  if (n < lut.max_exact) return base + n;
  int k = 0;
  for (int m = 0; m < lut.n_thr; ++m) k += (n >= lut.thr[m]) ? 1 : 0;
  int b = lut.max_exact + k;
  if (b > lut.n_side - 1) b = lut.n_side - 1;
  return base + b;
}

typedef __attribute__((address_space(3))) char lds_char;

// Streaming (non-temporal) global accesses for data this kernel touches exactly once: outputs and
// epilogue operands.  They should not push the operand panels that are being reused out of L2.
__device__ __forceinline__ void st_stream(bf16x4* p, bf16x4 v) {
  __builtin_nontemporal_store(__builtin_bit_cast(u32x2, v), reinterpret_cast<u32x2*>(p));
}
__device__ __forceinline__ void st_stream(f32x4* p, f32x4 v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ bf16x4 ld_stream(const bf16x4* p) {
  return __builtin_bit_cast(bf16x4, __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p)));
}
__device__ __forceinline__ f32x4 ld_stream(const f32x4* p) { return __builtin_nontemporal_load(p); }

// Direct global -> LDS copy (global_load_lds_dwordx4).  64 lanes x 16 bytes: lane L fetches 16 bytes at
// sbase + voff and they land at LDS address lds_addr + 16*L, so a wave fills 1 KB of contiguous LDS.
// lds_addr and sbase are wave-uniform.  The compiler does not know that this writes LDS: callers
// order it explicitly with s_waitcnt vmcnt(n) and a barrier before the data is read.
__device__ __forceinline__ void dma_1k(uint32_t lds_addr, const void* sbase, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff),
               "s"(sbase));
}

inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }
inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

}  // namespace t5mi
