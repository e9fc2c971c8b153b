// Reference-grade attention (paper Sec. 4 models): self-attention with the T5 relative-position
// bias, or cross-attention over a second sequence without bias or mask.  Any d_kv and sequence
// lengths, float32 or bf16 storage, float32 arithmetic.  One wavefront per query row (forward, dq)
// or per key row (dk, dv); scores live in LDS, never in HBM.
// With dropout of the attention probabilities (a.drop.on) the multiplier M of element
// ((b*H + h)*S + i, j) is regenerated wherever it is needed: O = (P o M) V, dV = (P o M)^T dO,
// dS = P o (M o (dO V^T) - rowsum(dO o O)); the softmax normaliser is that of the undropped P.
#include "kernels.h"

namespace t5mi {

namespace {

constexpr int AW = 4;  // waves per workgroup

template <typename T>
__device__ __forceinline__ float dot_row(const T* __restrict__ a, const T* __restrict__ b, int dk) {
  float s = 0.f;
  for (int c = 0; c < dk; ++c) s = fmaf(to_f32(a[c]), to_f32(b[c]), s);
  return s;
}

// grid.x = ceil(B*H*S / AW).  LDS: AW * Sk floats.
template <typename T>
__global__ __launch_bounds__(AW * 64) void attn_fwd_simple_kernel(AttnIO io, const float* __restrict__ diag,
                                                                  T* __restrict__ c, float* __restrict__ lse,
                                                                  AttnDims a) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * AW + wave;
  if (row >= (int64_t)a.B * a.H * a.S) return;
  const int i = (int)(row % a.S);
  const int h = (int)((row / a.S) % a.H);
  const int b = (int)(row / ((int64_t)a.S * a.H));
  const int I = a.H * a.dk;
  float* p = lds + wave * a.Sk;
  const T* q = (const T*)io.q + ((size_t)b * a.S + i) * io.ldq + h * a.dk;
  const T* kbase = (const T*)io.k + (size_t)b * a.Sk * io.ldkv + h * a.dk;
  const T* vbase = (const T*)io.v + (size_t)b * a.Sk * io.ldkv + h * a.dk;
  const float* dg = a.bias ? diag + (size_t)h * (2 * a.S - 1) + (a.S - 1) - i : nullptr;  // dg[j] = bias(j - i)
  const int jend = a.causal ? i + 1 : a.Sk;
  float m = -INFINITY;
  for (int j = lane; j < jend; j += 64) {
    float s = a.scale * dot_row(q, kbase + (size_t)j * io.ldkv, a.dk);
    if (a.bias) s += dg[j];
    p[j] = s;
    m = fmaxf(m, s);
  }
  m = wave_max(m);
  float l = 0.f;
  for (int j = lane; j < jend; j += 64) {
    const float e = __expf(p[j] - m);
    p[j] = e;
    l += e;
  }
  l = wave_sum(l);
  if (lane == 0) lse[row] = m + __logf(l);
  const float inv_l = 1.f / l;
  if (a.drop.on) {
    const uint32_t k1 = drop_row_key(a.drop, (uint32_t)row);
    for (int j = lane; j < jend; j += 64) p[j] *= drop_mult(a.drop, k1, (uint32_t)j);
  }
  // LDS writes above are read by other lanes of the same wave below
  __builtin_amdgcn_s_waitcnt(0);
  __builtin_amdgcn_wave_barrier();
  for (int ch = lane; ch < a.dk; ch += 64) {
    float o = 0.f;
    for (int j = 0; j < jend; ++j) o = fmaf(p[j], to_f32(vbase[(size_t)j * io.ldkv + ch]), o);
    c[((size_t)b * a.S + i) * I + h * a.dk + ch] = from_f32<T>(o * inv_l);
  }
}

// dq and (with bias) the per-diagonal bias gradient.  One wave per query row.
template <typename T>
__global__ __launch_bounds__(AW * 64) void attn_bwd_dq_simple_kernel(
    AttnIO io, const T* __restrict__ c, const T* __restrict__ dc, const float* __restrict__ diag,
    const float* __restrict__ lse, float* __restrict__ dvec, float* __restrict__ ddiag, AttnDims a) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * AW + wave;
  if (row >= (int64_t)a.B * a.H * a.S) return;
  const int i = (int)(row % a.S);
  const int h = (int)((row / a.S) % a.H);
  const int b = (int)(row / ((int64_t)a.S * a.H));
  const int I = a.H * a.dk;
  float* ds = lds + wave * a.Sk;
  const T* q = (const T*)io.q + ((size_t)b * a.S + i) * io.ldq + h * a.dk;
  const T* kbase = (const T*)io.k + (size_t)b * a.Sk * io.ldkv + h * a.dk;
  const T* vbase = (const T*)io.v + (size_t)b * a.Sk * io.ldkv + h * a.dk;
  const T* dor = dc + ((size_t)b * a.S + i) * I + h * a.dk;
  const T* orow = c + ((size_t)b * a.S + i) * I + h * a.dk;
  const int w = 2 * a.S - 1;
  const float* dg = a.bias ? diag + (size_t)h * w + (a.S - 1) - i : nullptr;
  float* ddg = a.bias ? ddiag + (size_t)h * w + (a.S - 1) - i : nullptr;
  float dsum = 0.f;
  for (int ch = lane; ch < a.dk; ch += 64) dsum += to_f32(dor[ch]) * to_f32(orow[ch]);
  dsum = wave_sum(dsum);
  if (lane == 0) dvec[row] = dsum;
  const float l = lse[row];
  const int jend = a.causal ? i + 1 : a.Sk;
  const uint32_t k1 = drop_row_key(a.drop, (uint32_t)row);
  for (int j = lane; j < jend; j += 64) {
    float s = a.scale * dot_row(q, kbase + (size_t)j * io.ldkv, a.dk);
    if (a.bias) s += dg[j];
    const float p = __expf(s - l);
    float dp = dot_row(dor, vbase + (size_t)j * io.ldkv, a.dk);
    if (a.drop.on) dp *= drop_mult(a.drop, k1, (uint32_t)j);
    const float d = p * (dp - dsum);
    ds[j] = d;
    if (a.bias) atomicAdd(ddg + j, d);
  }
  __builtin_amdgcn_s_waitcnt(0);
  __builtin_amdgcn_wave_barrier();
  T* dq = (T*)io.dq + ((size_t)b * a.S + i) * io.lddq + h * a.dk;
  for (int ch = lane; ch < a.dk; ch += 64) {
    float o = 0.f;
    for (int j = 0; j < jend; ++j) o = fmaf(ds[j], to_f32(kbase[(size_t)j * io.ldkv + ch]), o);
    dq[ch] = from_f32<T>(a.scale * o);
  }
}

// dk and dv.  One wave per key row; grid.x = ceil(B*H*Sk / AW); LDS: AW * 2 * S floats.
template <typename T>
__global__ __launch_bounds__(AW * 64) void attn_bwd_dkv_simple_kernel(
    AttnIO io, const T* __restrict__ dc, const float* __restrict__ diag, const float* __restrict__ lse,
    const float* __restrict__ dvec, AttnDims a) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * AW + wave;
  if (row >= (int64_t)a.B * a.H * a.Sk) return;
  const int j = (int)(row % a.Sk);
  const int h = (int)((row / a.Sk) % a.H);
  const int b = (int)(row / ((int64_t)a.Sk * a.H));
  const int I = a.H * a.dk;
  float* ps = lds + wave * 2 * a.S;
  float* dss = ps + a.S;
  const T* qbase = (const T*)io.q + (size_t)b * a.S * io.ldq + h * a.dk;
  const T* kr = (const T*)io.k + ((size_t)b * a.Sk + j) * io.ldkv + h * a.dk;
  const T* vr = (const T*)io.v + ((size_t)b * a.Sk + j) * io.ldkv + h * a.dk;
  const T* dobase = dc + (size_t)b * a.S * I + h * a.dk;
  const int w = 2 * a.S - 1;
  const float* dg = a.bias ? diag + (size_t)h * w + (a.S - 1) + j : nullptr;  // dg[-i] = bias(j - i)
  const size_t srow = ((size_t)b * a.H + h) * a.S;
  const int ibeg = a.causal ? j : 0;
  for (int i = ibeg + lane; i < a.S; i += 64) {
    float s = a.scale * dot_row(qbase + (size_t)i * io.ldq, kr, a.dk);
    if (a.bias) s += dg[-i];
    const float p = __expf(s - lse[srow + i]);
    const float dp = dot_row(dobase + (size_t)i * I, vr, a.dk);
    const float mk = a.drop.on ? drop_mult(a.drop, drop_row_key(a.drop, (uint32_t)(srow + i)), (uint32_t)j) : 1.f;
    ps[i] = p * mk;
    dss[i] = p * (dp * mk - dvec[srow + i]);
  }
  __builtin_amdgcn_s_waitcnt(0);
  __builtin_amdgcn_wave_barrier();
  T* dkr = (T*)io.dk + ((size_t)b * a.Sk + j) * io.lddkv + h * a.dk;
  T* dvr = (T*)io.dv + ((size_t)b * a.Sk + j) * io.lddkv + h * a.dk;
  for (int ch = lane; ch < a.dk; ch += 64) {
    float dv = 0.f, dk = 0.f;
    for (int i = ibeg; i < a.S; ++i) {
      dv = fmaf(ps[i], to_f32(dobase[(size_t)i * I + ch]), dv);
      dk = fmaf(dss[i], to_f32(qbase[(size_t)i * io.ldq + ch]), dk);
    }
    dkr[ch] = from_f32<T>(a.scale * dk);
    dvr[ch] = from_f32<T>(dv);
  }
}

__global__ void zero_diag_kernel(float* p, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

}  // namespace

hipError_t launch_attn_fwd_simple(const AttnIO& io, int type, const float* diag, void* c, float* lse,
                                  const AttnDims& a, hipStream_t st) {
  const int64_t rows = (int64_t)a.B * a.H * a.S;
  const int grid = ceil_div(rows, AW);
  const size_t lds = sizeof(float) * AW * a.Sk;
  if (type == IN_BF16)
    attn_fwd_simple_kernel<bf16><<<grid, AW * 64, lds, st>>>(io, diag, (bf16*)c, lse, a);
  else
    attn_fwd_simple_kernel<float><<<grid, AW * 64, lds, st>>>(io, diag, (float*)c, lse, a);
  return hipGetLastError();
}

hipError_t launch_attn_bwd_simple(const AttnIO& io, const void* c, const void* dc, int type,
                                  const float* diag, const float* lse, float* dvec, float* ddiag,
                                  const AttnDims& a, int zero_ddiag, hipStream_t st) {
  const int grid_q = ceil_div((int64_t)a.B * a.H * a.S, AW);
  const int grid_k = ceil_div((int64_t)a.B * a.H * a.Sk, AW);
  if (a.bias && zero_ddiag) {
    const int64_t nd = (int64_t)a.H * (2 * a.S - 1);
    zero_diag_kernel<<<ceil_div(nd, 256), 256, 0, st>>>(ddiag, nd);
  }
  const size_t lds_q = sizeof(float) * AW * a.Sk, lds_k = sizeof(float) * AW * 2 * a.S;
  if (type == IN_BF16) {
    attn_bwd_dq_simple_kernel<bf16><<<grid_q, AW * 64, lds_q, st>>>(io, (const bf16*)c, (const bf16*)dc, diag, lse,
                                                                    dvec, ddiag, a);
    attn_bwd_dkv_simple_kernel<bf16><<<grid_k, AW * 64, lds_k, st>>>(io, (const bf16*)dc, diag, lse, dvec, a);
  } else {
    attn_bwd_dq_simple_kernel<float><<<grid_q, AW * 64, lds_q, st>>>(io, (const float*)c, (const float*)dc, diag,
                                                                     lse, dvec, ddiag, a);
    attn_bwd_dkv_simple_kernel<float><<<grid_k, AW * 64, lds_k, st>>>(io, (const float*)dc, diag, lse, dvec, a);
  }
  return hipGetLastError();
}

}  // namespace t5mi
