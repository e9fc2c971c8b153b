// Reference-grade self-attention with the T5 relative-position bias (paper Sec. 4 models), any
// d_kv and sequence length, float32 or bf16 storage, float32 arithmetic.  One wavefront per query
// row (forward, dq) or per key row (dk, dv); scores live in LDS, never in HBM.
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

// grid.x = ceil(B*H*S / AW).  LDS: AW * S floats.
template <typename T>
__global__ __launch_bounds__(AW * 64) void attn_fwd_simple_kernel(const T* __restrict__ qkv,
                                                                  const float* __restrict__ diag,
                                                                  T* __restrict__ c, float* __restrict__ lse,
                                                                  AttnDims a) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * AW + wave;
  if (row >= (int64_t)a.B * a.H * a.S) return;
  const int i = (int)(row % a.S);
  const int h = (int)((row / a.S) % a.H);
  const int b = (int)(row / ((int64_t)a.S * a.H));
  const int I = a.H * a.dk, ld = 3 * I;
  float* p = lds + wave * a.S;
  const T* q = qkv + ((size_t)b * a.S + i) * ld + h * a.dk;
  const T* kbase = qkv + (size_t)b * a.S * ld + I + h * a.dk;
  const T* vbase = kbase + I;
  const float* dg = diag + (size_t)h * (2 * a.S - 1) + (a.S - 1) - i;  // dg[j] = bias(j - i)
  const int jend = a.causal ? i + 1 : a.S;
  float m = -INFINITY;
  for (int j = lane; j < jend; j += 64) {
    const float s = a.scale * dot_row(q, kbase + (size_t)j * ld, a.dk) + dg[j];
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
  // LDS writes above are read by other lanes of the same wave below
  __builtin_amdgcn_s_waitcnt(0);
  __builtin_amdgcn_wave_barrier();
  for (int ch = lane; ch < a.dk; ch += 64) {
    float o = 0.f;
    for (int j = 0; j < jend; ++j) o = fmaf(p[j], to_f32(vbase[(size_t)j * ld + ch]), o);
    c[((size_t)b * a.S + i) * I + h * a.dk + ch] = from_f32<T>(o * inv_l);
  }
}

// dq and the per-diagonal bias gradient.  One wave per query row.
template <typename T>
__global__ __launch_bounds__(AW * 64) void attn_bwd_dq_simple_kernel(
    const T* __restrict__ qkv, const T* __restrict__ c, const T* __restrict__ dc,
    const float* __restrict__ diag, const float* __restrict__ lse, float* __restrict__ dvec,
    T* __restrict__ dqkv, float* __restrict__ ddiag, AttnDims a) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * AW + wave;
  if (row >= (int64_t)a.B * a.H * a.S) return;
  const int i = (int)(row % a.S);
  const int h = (int)((row / a.S) % a.H);
  const int b = (int)(row / ((int64_t)a.S * a.H));
  const int I = a.H * a.dk, ld = 3 * I;
  float* ds = lds + wave * a.S;
  const T* q = qkv + ((size_t)b * a.S + i) * ld + h * a.dk;
  const T* kbase = qkv + (size_t)b * a.S * ld + I + h * a.dk;
  const T* vbase = kbase + I;
  const T* dor = dc + ((size_t)b * a.S + i) * I + h * a.dk;
  const T* orow = c + ((size_t)b * a.S + i) * I + h * a.dk;
  const int w = 2 * a.S - 1;
  const float* dg = diag + (size_t)h * w + (a.S - 1) - i;
  float* ddg = ddiag + (size_t)h * w + (a.S - 1) - i;
  float dsum = 0.f;
  for (int ch = lane; ch < a.dk; ch += 64) dsum += to_f32(dor[ch]) * to_f32(orow[ch]);
  dsum = wave_sum(dsum);
  if (lane == 0) dvec[row] = dsum;
  const float l = lse[row];
  const int jend = a.causal ? i + 1 : a.S;
  for (int j = lane; j < jend; j += 64) {
    const float s = a.scale * dot_row(q, kbase + (size_t)j * ld, a.dk) + dg[j];
    const float p = __expf(s - l);
    const float dp = dot_row(dor, vbase + (size_t)j * ld, a.dk);
    const float d = p * (dp - dsum);
    ds[j] = d;
    atomicAdd(ddg + j, d);
  }
  __builtin_amdgcn_s_waitcnt(0);
  __builtin_amdgcn_wave_barrier();
  for (int ch = lane; ch < a.dk; ch += 64) {
    float o = 0.f;
    for (int j = 0; j < jend; ++j) o = fmaf(ds[j], to_f32(kbase[(size_t)j * ld + ch]), o);
    dqkv[((size_t)b * a.S + i) * ld + h * a.dk + ch] = from_f32<T>(a.scale * o);
  }
}

// dk and dv.  One wave per key row; LDS: AW * 2 * S floats.
template <typename T>
__global__ __launch_bounds__(AW * 64) void attn_bwd_dkv_simple_kernel(
    const T* __restrict__ qkv, const T* __restrict__ dc, const float* __restrict__ diag,
    const float* __restrict__ lse, const float* __restrict__ dvec, T* __restrict__ dqkv, AttnDims a) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = (int64_t)blockIdx.x * AW + wave;
  if (row >= (int64_t)a.B * a.H * a.S) return;
  const int j = (int)(row % a.S);
  const int h = (int)((row / a.S) % a.H);
  const int b = (int)(row / ((int64_t)a.S * a.H));
  const int I = a.H * a.dk, ld = 3 * I;
  float* ps = lds + wave * 2 * a.S;
  float* dss = ps + a.S;
  const T* qbase = qkv + (size_t)b * a.S * ld + h * a.dk;
  const T* kr = qbase + I + (size_t)j * ld;
  const T* vr = kr + I;
  const T* dobase = dc + (size_t)b * a.S * I + h * a.dk;
  const int w = 2 * a.S - 1;
  const float* dg = diag + (size_t)h * w + (a.S - 1) + j;  // dg[-i] = bias(j - i)
  const size_t srow = ((size_t)b * a.H + h) * a.S;
  const int ibeg = a.causal ? j : 0;
  for (int i = ibeg + lane; i < a.S; i += 64) {
    const float s = a.scale * dot_row(qbase + (size_t)i * ld, kr, a.dk) + dg[-i];
    const float p = __expf(s - lse[srow + i]);
    const float dp = dot_row(dobase + (size_t)i * I, vr, a.dk);
    ps[i] = p;
    dss[i] = p * (dp - dvec[srow + i]);
  }
  __builtin_amdgcn_s_waitcnt(0);
  __builtin_amdgcn_wave_barrier();
  for (int ch = lane; ch < a.dk; ch += 64) {
    float dv = 0.f, dk = 0.f;
    for (int i = ibeg; i < a.S; ++i) {
      dv = fmaf(ps[i], to_f32(dobase[(size_t)i * I + ch]), dv);
      dk = fmaf(dss[i], to_f32(qbase[(size_t)i * ld + ch]), dk);
    }
    T* out = dqkv + ((size_t)b * a.S + j) * ld + h * a.dk + ch;
    out[I] = from_f32<T>(a.scale * dk);
    out[2 * I] = from_f32<T>(dv);
  }
}

__global__ void zero_f32_kernel(float* p, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

}  // namespace

hipError_t launch_attn_fwd_simple(const void* qkv, int type, const float* diag, void* c, float* lse,
                                  const AttnDims& a, hipStream_t st) {
  const int64_t rows = (int64_t)a.B * a.H * a.S;
  const int grid = ceil_div(rows, AW);
  const size_t lds = sizeof(float) * AW * a.S;
  if (type == IN_BF16)
    attn_fwd_simple_kernel<bf16><<<grid, AW * 64, lds, st>>>((const bf16*)qkv, diag, (bf16*)c, lse, a);
  else
    attn_fwd_simple_kernel<float><<<grid, AW * 64, lds, st>>>((const float*)qkv, diag, (float*)c, lse, a);
  return hipGetLastError();
}

hipError_t launch_attn_bwd_simple(const void* qkv, const void* c, const void* dc, int type,
                                  const float* diag, const float* lse, float* dvec, void* dqkv,
                                  float* ddiag, const AttnDims& a, hipStream_t st) {
  const int64_t rows = (int64_t)a.B * a.H * a.S;
  const int grid = ceil_div(rows, AW);
  const int64_t nd = (int64_t)a.H * (2 * a.S - 1);
  zero_f32_kernel<<<ceil_div(nd, 256), 256, 0, st>>>(ddiag, nd);
  if (type == IN_BF16) {
    attn_bwd_dq_simple_kernel<bf16><<<grid, AW * 64, sizeof(float) * AW * a.S, st>>>(
        (const bf16*)qkv, (const bf16*)c, (const bf16*)dc, diag, lse, dvec, (bf16*)dqkv, ddiag, a);
    attn_bwd_dkv_simple_kernel<bf16><<<grid, AW * 64, sizeof(float) * AW * 2 * a.S, st>>>(
        (const bf16*)qkv, (const bf16*)dc, diag, lse, dvec, (bf16*)dqkv, a);
  } else {
    attn_bwd_dq_simple_kernel<float><<<grid, AW * 64, sizeof(float) * AW * a.S, st>>>(
        (const float*)qkv, (const float*)c, (const float*)dc, diag, lse, dvec, (float*)dqkv, ddiag, a);
    attn_bwd_dkv_simple_kernel<float><<<grid, AW * 64, sizeof(float) * AW * 2 * a.S, st>>>(
        (const float*)qkv, (const float*)dc, diag, lse, dvec, (float*)dqkv, a);
  }
  return hipGetLastError();
}

}  // namespace t5mi
