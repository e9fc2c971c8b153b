// T5 layer norm (scale-only RMS norm, the norm of the models in paper Sec. 4): forward and backward.
// HBM-bound: one wavefront per token row, 16-byte loads, float32 statistics, wave reductions.
#include "kernels.h"

namespace t5mi {

namespace {

template <typename T, int VEC>
__device__ __forceinline__ void load_vec(const T* __restrict__ p, float (&v)[VEC]) {
  if constexpr (VEC == 1) {
    v[0] = to_f32(p[0]);
  } else if constexpr (sizeof(T) == 2) {
    bf16x8 t = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (float)t[i];
  } else {
    f32x4 a = *reinterpret_cast<const f32x4*>(p);
    f32x4 b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[i] = a[i]; v[4 + i] = b[i]; }
  }
}

template <typename T, int VEC>
__device__ __forceinline__ void store_vec(T* __restrict__ p, const float (&v)[VEC]) {
  if constexpr (VEC == 1) {
    p[0] = from_f32<T>(v[0]);
  } else if constexpr (sizeof(T) == 2) {
    bf16x8 t;
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = (bf16)v[i];
    *reinterpret_cast<bf16x8*>(p) = t;
  } else {
    f32x4 a, b;
#pragma unroll
    for (int i = 0; i < 4; ++i) { a[i] = v[i]; b[i] = v[4 + i]; }
    *reinterpret_cast<f32x4*>(p) = a;
    *reinterpret_cast<f32x4*>(p + 4) = b;
  }
}

constexpr int kNormWaves = 4;

// NV > 0: the row (NV vectors of VEC columns per lane, d <= 64 * VEC * NV) stays in registers between the sum of
// squares and the scaling, so that it is read once; read a second time it came from the fabric again (the counters
// showed twice the algorithmic bytes).  NV == 0: any width, two passes over the row.
template <typename TX, typename TO, int VEC, int NV>
__global__ __launch_bounds__(kNormWaves * 64) void rmsnorm_fwd_kernel(
    const TX* __restrict__ x, const TO* __restrict__ g, TO* __restrict__ n, float* __restrict__ r, int T,
    int d, float eps) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const float inv_d = 1.f / (float)d;
  for (int row = blockIdx.x * kNormWaves + wave; row < T; row += gridDim.x * kNormWaves) {
    const TX* xr = x + (size_t)row * d;
    TO* nr = n + (size_t)row * d;
    float ss = 0.f;
    if constexpr (NV > 0) {
      float xv[NV][VEC];
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int c = (j * 64 + lane) * VEC;
        if (c < d) {
          load_vec<TX, VEC>(xr + c, xv[j]);
#pragma unroll
          for (int i = 0; i < VEC; ++i) ss += xv[j][i] * xv[j][i];
        }
      }
      ss = wave_sum(ss);
      const float rr = rsqrtf(ss * inv_d + eps);
      if (lane == 0) r[row] = rr;
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int c = (j * 64 + lane) * VEC;
        if (c < d) {
          float gg[VEC], o[VEC];
          load_vec<TO, VEC>(g + c, gg);
#pragma unroll
          for (int i = 0; i < VEC; ++i) o[i] = xv[j][i] * rr * gg[i];
          store_vec<TO, VEC>(nr + c, o);
        }
      }
    } else {
      for (int c = lane * VEC; c < d; c += 64 * VEC) {
        float v[VEC];
        load_vec<TX, VEC>(xr + c, v);
#pragma unroll
        for (int i = 0; i < VEC; ++i) ss += v[i] * v[i];
      }
      ss = wave_sum(ss);
      const float rr = rsqrtf(ss * inv_d + eps);
      if (lane == 0) r[row] = rr;
      for (int c = lane * VEC; c < d; c += 64 * VEC) {
        float v[VEC], gg[VEC], o[VEC];
        load_vec<TX, VEC>(xr + c, v);
        load_vec<TO, VEC>(g + c, gg);
#pragma unroll
        for (int i = 0; i < VEC; ++i) o[i] = v[i] * rr * gg[i];
        store_vec<TO, VEC>(nr + c, o);
      }
    }
  }
}

// Backward.  Each wave walks rows; lane keeps float32 partial sums of dg for its columns
// (NV vectors of VEC columns); the workgroup's four waves are combined through LDS and written to
// dg_partial[blockIdx.x][d]; rmsnorm_dg_reduce_kernel sums the partial rows in a fixed order.
template <typename TX, typename TG, typename TR, typename TL, int VEC, int NV>
__global__ __launch_bounds__(kNormWaves * 64) void rmsnorm_bwd_kernel(
    const TX* __restrict__ x, const TG* __restrict__ g, const float* __restrict__ r,
    const float* __restrict__ dn, const TR* __restrict__ resid, float* __restrict__ out_f32,
    TL* __restrict__ out_lp, float* __restrict__ dg_partial, int T, int d) {
  extern __shared__ float lds_dg[];  // [kNormWaves][d]
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const float inv_d = 1.f / (float)d;
  float dgacc[NV][VEC];
#pragma unroll
  for (int j = 0; j < NV; ++j)
#pragma unroll
    for (int i = 0; i < VEC; ++i) dgacc[j][i] = 0.f;

  for (int row = blockIdx.x * kNormWaves + wave; row < T; row += gridDim.x * kNormWaves) {
    const TX* xr = x + (size_t)row * d;
    const float* dnr = dn + (size_t)row * d;
    const float rr = r[row];
    float dot = 0.f;
    // x * r and dn * g of the row stay in registers for the second pass: x and dn are read once
    float xh[NV][VEC], dgn[NV][VEC];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int c = (j * 64 + lane) * VEC;
      if (c < d) {
        float xv[VEC], dv[VEC], gv[VEC];
        load_vec<TX, VEC>(xr + c, xv);
        load_vec<float, VEC>(dnr + c, dv);
        load_vec<TG, VEC>(g + c, gv);
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          xh[j][i] = xv[i] * rr;
          dgn[j][i] = dv[i] * gv[i];
          dgacc[j][i] += dv[i] * xh[j][i];
          dot += dgn[j][i] * xh[j][i];
        }
      }
    }
    dot = wave_sum(dot) * inv_d;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int c = (j * 64 + lane) * VEC;
      if (c < d) {
        float rv[VEC], o[VEC];
        if (resid) {
          load_vec<TR, VEC>(resid + (size_t)row * d + c, rv);
        } else {
#pragma unroll
          for (int i = 0; i < VEC; ++i) rv[i] = 0.f;
        }
#pragma unroll
        for (int i = 0; i < VEC; ++i) o[i] = rv[i] + rr * (dgn[j][i] - xh[j][i] * dot);
        if (out_f32) store_vec<float, VEC>(out_f32 + (size_t)row * d + c, o);
        if (out_lp) store_vec<TL, VEC>(out_lp + (size_t)row * d + c, o);
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int c = (j * 64 + lane) * VEC;
    if (c < d) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) lds_dg[wave * d + c + i] = dgacc[j][i];
    }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < d; c += kNormWaves * 64) {
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < kNormWaves; ++w) s += lds_dg[w * d + c];
    dg_partial[(size_t)blockIdx.x * d + c] = s;
  }
}

// 1024 threads = 32 columns x 32 row slices; the slices meet in LDS in a fixed order.
__global__ __launch_bounds__(1024) void rmsnorm_dg_reduce_kernel(const float* __restrict__ part, int nrows, int d,
                                                                 float* __restrict__ dg, int accumulate) {
  __shared__ float red[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int c = blockIdx.x * 32 + tx;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (c < d) {
    int i = ty;
    for (; i + 96 < nrows; i += 128) {
      s0 += part[(size_t)i * d + c];
      s1 += part[(size_t)(i + 32) * d + c];
      s2 += part[(size_t)(i + 64) * d + c];
      s3 += part[(size_t)(i + 96) * d + c];
    }
    for (; i < nrows; i += 32) s0 += part[(size_t)i * d + c];
  }
  red[ty][tx] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (ty == 0 && c < d) {
    float t = 0.f;
#pragma unroll
    for (int k = 0; k < 32; ++k) t += red[k][tx];
    dg[c] = accumulate ? dg[c] + t : t;
  }
}

template <typename TX, typename TO>
hipError_t fwd_dispatch(const void* x, const void* g, void* n, float* r, int T, int d, float eps,
                        hipStream_t st) {
  int grid = ceil_div(T, kNormWaves);
  if (grid > 8192) grid = 8192;
#define T5MI_FWD(VEC, NV)                                                                                          \
  rmsnorm_fwd_kernel<TX, TO, VEC, NV><<<grid, kNormWaves * 64, 0, st>>>((const TX*)x, (const TO*)g, (TO*)n, r, T, d, \
                                                                      eps)
  if (d % 8 == 0) {
    const int nv = ceil_div(d, 512);
    if (nv <= 1) T5MI_FWD(8, 1);
    else if (nv <= 2) T5MI_FWD(8, 2);
    else if (nv <= 4) T5MI_FWD(8, 4);
    else if (nv <= 8) T5MI_FWD(8, 8);
    else T5MI_FWD(8, 0);
  } else {
    T5MI_FWD(1, 0);
  }
#undef T5MI_FWD
  return hipGetLastError();
}

template <typename TX, typename TG, typename TR, typename TL, int VEC, int NV>
hipError_t bwd_launch(const void* x, const void* g, const float* r, const float* dn, const void* resid,
                      float* out_f32, void* out_lp, float* dg_partial, int T, int d, int grid,
                      hipStream_t st) {
  rmsnorm_bwd_kernel<TX, TG, TR, TL, VEC, NV><<<grid, kNormWaves * 64, sizeof(float) * kNormWaves * d, st>>>(
      (const TX*)x, (const TG*)g, r, dn, (const TR*)resid, out_f32, (TL*)out_lp, dg_partial, T, d);
  return hipGetLastError();
}

template <typename TX, typename TG, typename TR, typename TL>
hipError_t bwd_dispatch(const void* x, const void* g, const float* r, const float* dn, const void* resid,
                        float* out_f32, void* out_lp, float* dg_partial, int T, int d, int grid,
                        hipStream_t st) {
#define T5MI_BWD(VEC, NV) \
  return bwd_launch<TX, TG, TR, TL, VEC, NV>(x, g, r, dn, resid, out_f32, out_lp, dg_partial, T, d, grid, st)
  if (d % 8 == 0) {
    const int nv = ceil_div(d, 512);
    if (nv <= 1) T5MI_BWD(8, 1);
    if (nv <= 2) T5MI_BWD(8, 2);
    if (nv <= 4) T5MI_BWD(8, 4);
    if (nv <= 8) T5MI_BWD(8, 8);
    if (nv <= 16) T5MI_BWD(8, 16);
    return hipErrorInvalidValue;
  }
  const int nv = ceil_div(d, 64);
  if (nv <= 4) T5MI_BWD(1, 4);
  if (nv <= 16) T5MI_BWD(1, 16);
  return hipErrorInvalidValue;
#undef T5MI_BWD
}

}  // namespace

hipError_t launch_rmsnorm_fwd(const void* x, int x_type, const void* g, void* n, int out_type, float* r,
                              int T, int d, float eps, hipStream_t st) {
  if (out_type == IN_BF16) {
    if (x_type == IN_BF16) return fwd_dispatch<bf16, bf16>(x, g, n, r, T, d, eps, st);
    return fwd_dispatch<float, bf16>(x, g, n, r, T, d, eps, st);
  }
  if (x_type == IN_BF16) return hipErrorInvalidValue;
  return fwd_dispatch<float, float>(x, g, n, r, T, d, eps, st);
}

int rmsnorm_bwd_partial_rows(int T) {
  int grid = ceil_div(T, 4 * kNormWaves);
  if (grid > 1024) grid = 1024;
  if (grid < 1) grid = 1;
  return grid;
}

// Supported type combinations: (x, g, resid, lp) =
//   (f32, bf16, bf16, bf16)  norm 2 of the bf16 block: x = h, resid = dy, outputs dh f32 + bf16
//   (bf16, bf16, f32, bf16)  norm 1 of the bf16 block: x = x, resid = dh, output dx bf16
//   (f32, bf16, f32, bf16)   cross-attention norm of the bf16 decoder block: x = h, resid = dh2
//   (f32, f32, f32, f32)     both norms of the float32 block
hipError_t launch_rmsnorm_bwd(const void* x, int x_type, const void* g, int g_type, const float* r,
                              const float* dn, const void* resid, int resid_type, float* out_f32,
                              void* out_lp, int lp_type, float* dg, float* dg_partial, int accumulate,
                              int T, int d, hipStream_t st) {
  const int grid = rmsnorm_bwd_partial_rows(T);
  hipError_t e;
  if (x_type == IN_F32 && g_type == IN_BF16 && resid_type == IN_BF16 && lp_type == IN_BF16)
    e = bwd_dispatch<float, bf16, bf16, bf16>(x, g, r, dn, resid, out_f32, out_lp, dg_partial, T, d, grid, st);
  else if (x_type == IN_BF16 && g_type == IN_BF16 && resid_type == IN_F32 && lp_type == IN_BF16)
    e = bwd_dispatch<bf16, bf16, float, bf16>(x, g, r, dn, resid, out_f32, out_lp, dg_partial, T, d, grid, st);
  else if (x_type == IN_F32 && g_type == IN_BF16 && resid_type == IN_F32 && lp_type == IN_BF16)
    e = bwd_dispatch<float, bf16, float, bf16>(x, g, r, dn, resid, out_f32, out_lp, dg_partial, T, d, grid, st);
  else if (x_type == IN_F32 && g_type == IN_F32 && resid_type == IN_F32 && lp_type == IN_F32)
    e = bwd_dispatch<float, float, float, float>(x, g, r, dn, resid, out_f32, out_lp, dg_partial, T, d, grid,
                                                 st);
  else
    return hipErrorInvalidValue;
  if (e != hipSuccess) return e;
  rmsnorm_dg_reduce_kernel<<<ceil_div(d, 32), 1024, 0, st>>>(dg_partial, grid, d, dg, accumulate);
  return hipGetLastError();
}

}  // namespace t5mi
