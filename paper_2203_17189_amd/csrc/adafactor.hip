// Adafactor with factored second moments and update clipping (the optimizer of the T5 models in
// paper Sec. 4).  HBM-bound: float32, 16-byte loads, wave reductions, deterministic two-stage sums.
//
// Factored tensor [R,C], tiles of 64 rows x 256 columns:
//   stats     : per-tile row sums and column sums of G*G          -> rowpart[tc][R], colpart[tr][C]
//   finalize  : v_row, v_col EMA; cfac_j = rsqrt(v_col_j); consumers form rsqrt(v_row_i / mean v_row)
//   norms     : per-tile sums of U*U (U = G rfac cfac) and of W*W -> part[2][tiles]
//   coef      : coef = lr * max(eps2, RMS(W)) / max(1, RMS(U)/clip)
//   apply     : W -= coef * U   (+ optional bf16 copy)
// Unfactored tensors use the same skeleton with v_full updated elementwise in the first pass.
#include "kernels.h"

namespace t5mi {

namespace {

constexpr int TR = 64;    // tile rows
constexpr int TCV = 256;  // tile cols when vectorised (64 lanes x 4)

struct AfWs {
  float* rowpart;  // [ntc][R]
  float* colpart;  // [ntr][C]
  float* part_u;   // [ntiles]
  float* part_w;   // [ntiles]
  float* rfac;     // [R]
  float* cfac;     // [C]
  float* scal;     // [4]: 0 = coef
};

template <int VEC>
__device__ __forceinline__ void ldv(const float* __restrict__ p, float (&v)[VEC]) {
  if constexpr (VEC == 4) {
    f32x4 t = *reinterpret_cast<const f32x4*>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = t[i];
  } else {
    v[0] = p[0];
  }
}
template <int VEC>
__device__ __forceinline__ void stv(float* __restrict__ p, const float (&v)[VEC]) {
  if constexpr (VEC == 4) {
    f32x4 t;
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = v[i];
    *reinterpret_cast<f32x4*>(p) = t;
  } else {
    p[0] = v[0];
  }
}

// grid (ntc, ntr), 256 threads.  Wave w takes rows w, w+4, ... of the tile; lanes span the columns.
template <int VEC>
__global__ __launch_bounds__(256) void af_stats_kernel(const float* __restrict__ g, int64_t R, int64_t C,
                                                       AfWs ws) {
  __shared__ float colred[4][64 * VEC];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c0 = (int64_t)blockIdx.x * 64 * VEC + lane * VEC;
  const int64_t r0 = (int64_t)blockIdx.y * TR;
  float csum[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) csum[i] = 0.f;
  for (int rr = wave; rr < TR; rr += 4) {
    const int64_t r = r0 + rr;
    if (r >= R) break;
    float rs = 0.f;
    if (c0 < C) {
      float v[VEC];
      ldv<VEC>(g + r * C + c0, v);
#pragma unroll
      for (int i = 0; i < VEC; ++i) {
        const float q = v[i] * v[i];
        csum[i] += q;
        rs += q;
      }
    }
    rs = wave_sum(rs);
    if (lane == 0) ws.rowpart[(int64_t)blockIdx.x * R + r] = rs;
  }
#pragma unroll
  for (int i = 0; i < VEC; ++i) colred[wave][lane * VEC + i] = csum[i];
  __syncthreads();
  for (int t = threadIdx.x; t < 64 * VEC; t += 256) {
    const int64_t c = (int64_t)blockIdx.x * 64 * VEC + t;
    if (c < C) ws.colpart[(int64_t)blockIdx.y * C + c] = colred[0][t] + colred[1][t] + colred[2][t] + colred[3][t];
  }
}

// One thread per row and per column: folds the tile partials into the second-moment vectors.
// cfac_j = rsqrt(v_col_j); the row factor needs mean(v_row) and is formed by the consumers.
__global__ __launch_bounds__(256) void af_finalize_kernel(float* __restrict__ v_row, float* __restrict__ v_col,
                                                          int64_t R, int64_t C, int ntc, int ntr, float beta2,
                                                          float eps1, AfWs ws) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx < R) {
    float s = 0.f;
    for (int t = 0; t < ntc; ++t) s += ws.rowpart[(int64_t)t * R + idx];
    v_row[idx] = beta2 * v_row[idx] + (1.f - beta2) * (s / (float)C + eps1);
  } else if (idx < R + C) {
    const int64_t j = idx - R;
    float s = 0.f;
    for (int t = 0; t < ntr; ++t) s += ws.colpart[(int64_t)t * C + j];
    const float vc = beta2 * v_col[j] + (1.f - beta2) * (s / (float)R + eps1);
    v_col[j] = vc;
    ws.cfac[j] = rsqrtf(vc);
  }
}

// mean(v_row) in a fixed order, by a whole workgroup of 256 threads (every workgroup gets the same value).
__device__ __forceinline__ float af_mean_vrow(const float* __restrict__ v_row, int64_t R, float* red) {
  float s = 0.f;
  for (int64_t i = threadIdx.x; i < R; i += 256) s += v_row[i];
  return block_sum<4>(s, red) / (float)R;
}

// Per-tile sums of U*U and W*W.  FACT: U = g rfac cfac.  !FACT: updates v_full and U = g rsqrt(v).
template <int VEC, bool FACT>
__global__ __launch_bounds__(256) void af_norms_kernel(const float* __restrict__ g, const float* __restrict__ w,
                                                       float* __restrict__ v_full, const float* __restrict__ v_row,
                                                       int64_t R, int64_t C, float beta2, float eps1, AfWs ws) {
  __shared__ float red[12];
  float inv_mean = 1.f;
  if constexpr (FACT) {
    const float mean_vr = af_mean_vrow(v_row, R, red + 8);
    inv_mean = 1.f / mean_vr;
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) ws.scal[1] = inv_mean;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c0 = (int64_t)blockIdx.x * 64 * VEC + lane * VEC;
  const int64_t r0 = (int64_t)blockIdx.y * TR;
  float su = 0.f, sw = 0.f;
  if (c0 < C) {
    float cf[VEC];
    if constexpr (FACT) ldv<VEC>(ws.cfac + c0, cf);
    for (int rr = wave; rr < TR; rr += 4) {
      const int64_t r = r0 + rr;
      if (r >= R) break;
      float gv[VEC], wv[VEC];
      ldv<VEC>(g + r * C + c0, gv);
      ldv<VEC>(w + r * C + c0, wv);
      if constexpr (FACT) {
        const float rf = rsqrtf(v_row[r] * inv_mean);
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          const float u = gv[i] * rf * cf[i];
          su += u * u;
          sw += wv[i] * wv[i];
        }
      } else {
        float vv[VEC];
        ldv<VEC>(v_full + r * C + c0, vv);
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          vv[i] = beta2 * vv[i] + (1.f - beta2) * (gv[i] * gv[i] + eps1);
          const float u = gv[i] * rsqrtf(vv[i]);
          su += u * u;
          sw += wv[i] * wv[i];
        }
        stv<VEC>(v_full + r * C + c0, vv);
      }
    }
  }
  su = block_sum<4>(su, red);
  sw = block_sum<4>(sw, red + 4);
  if (threadIdx.x == 0) {
    const int64_t tile = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
    ws.part_u[tile] = su;
    ws.part_w[tile] = sw;
  }
}

__global__ __launch_bounds__(1024) void af_coef_kernel(int64_t ntiles, double count, adafactor_cfg c, AfWs ws) {
  __shared__ float red[32];
  float su = 0.f, sw = 0.f;
  for (int64_t i = threadIdx.x; i < ntiles; i += 1024) {
    su += ws.part_u[i];
    sw += ws.part_w[i];
  }
  su = block_sum<16>(su, red);
  sw = block_sum<16>(sw, red + 16);
  if (threadIdx.x == 0) {
    const float rms_u = sqrtf(su / (float)count), rms_w = sqrtf(sw / (float)count);
    float alpha = c.lr;
    if (c.scale_by_param) alpha *= fmaxf(c.eps2, rms_w);
    ws.scal[0] = alpha / fmaxf(1.f, rms_u / c.clip);
  }
}

template <int VEC, bool FACT>
__global__ __launch_bounds__(256) void af_apply_kernel(float* __restrict__ w, const float* __restrict__ g,
                                                       const float* __restrict__ v_full, const float* __restrict__ v_row,
                                                       bf16* __restrict__ lp, int64_t R, int64_t C, AfWs ws) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c0 = (int64_t)blockIdx.x * 64 * VEC + lane * VEC;
  const int64_t r0 = (int64_t)blockIdx.y * TR;
  if (c0 >= C) return;
  const float coef = ws.scal[0];
  float cf[VEC];
  if constexpr (FACT) ldv<VEC>(ws.cfac + c0, cf);
  for (int rr = wave; rr < TR; rr += 4) {
    const int64_t r = r0 + rr;
    if (r >= R) break;
    float gv[VEC], wv[VEC];
    ldv<VEC>(g + r * C + c0, gv);
    ldv<VEC>(w + r * C + c0, wv);
    if constexpr (FACT) {
      const float rf = rsqrtf(v_row[r] * ws.scal[1]) * coef;
#pragma unroll
      for (int i = 0; i < VEC; ++i) wv[i] -= gv[i] * rf * cf[i];
    } else {
      float vv[VEC];
      ldv<VEC>(v_full + r * C + c0, vv);
#pragma unroll
      for (int i = 0; i < VEC; ++i) wv[i] -= coef * gv[i] * rsqrtf(vv[i]);
    }
    stv<VEC>(w + r * C + c0, wv);
    if (lp) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) lp[r * C + c0 + i] = (bf16)wv[i];
    }
  }
}

struct AfGeom {
  int vec, ntc, ntr;
  int64_t ntiles;
};
AfGeom geom(int64_t R, int64_t C) {
  AfGeom g;
  g.vec = (C % 4 == 0) ? 4 : 1;
  g.ntc = ceil_div(C, 64 * g.vec);
  g.ntr = ceil_div(R, TR);
  g.ntiles = (int64_t)g.ntc * g.ntr;
  return g;
}
AfWs carve(void* ws, int64_t R, int64_t C, const AfGeom& g) {
  char* p = (char*)ws;
  AfWs w;
  auto take = [&](size_t n) { float* r = (float*)p; p += align_up(n * sizeof(float)); return r; };
  w.rowpart = take((size_t)g.ntc * R);
  w.colpart = take((size_t)g.ntr * C);
  w.part_u = take(g.ntiles);
  w.part_w = take(g.ntiles);
  w.rfac = take(R);
  w.cfac = take(C);
  w.scal = take(4);
  return w;
}

}  // namespace

size_t adafactor_ws_bytes(int64_t R, int64_t C, int factored) {
  (void)factored;
  const AfGeom g = geom(R, C);
  size_t n = 0;
  n += align_up((size_t)g.ntc * R * 4) + align_up((size_t)g.ntr * C * 4);
  n += 2 * align_up((size_t)g.ntiles * 4) + align_up(R * 4) + align_up(C * 4) + align_up(16);
  return n;
}

hipError_t launch_adafactor(float* param, const float* grad, float* v_row, float* v_col, float* v_full,
                            int64_t R, int64_t C, int factored, const adafactor_cfg& c, void* bf16_out,
                            void* wsp, hipStream_t st) {
  const AfGeom g = geom(R, C);
  const AfWs ws = carve(wsp, R, C, g);
  const float beta2 = (float)(1.0 - pow((double)c.step, -(double)c.decay_pow));
  const dim3 grid(g.ntc, g.ntr);
  hipError_t e;
#define T5MI_AF(K, ...)                                                   \
  do {                                                                    \
    if (g.vec == 4) K<4, __VA_ARGS__; else K<1, __VA_ARGS__;              \
    if ((e = hipGetLastError()) != hipSuccess) return e;                  \
  } while (0)
  if (factored) {
    if (g.vec == 4) af_stats_kernel<4><<<grid, 256, 0, st>>>(grad, R, C, ws);
    else af_stats_kernel<1><<<grid, 256, 0, st>>>(grad, R, C, ws);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    af_finalize_kernel<<<ceil_div(R + C, 256), 256, 0, st>>>(v_row, v_col, R, C, g.ntc, g.ntr, beta2, c.eps1, ws);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    T5MI_AF(af_norms_kernel, true><<<grid, 256, 0, st>>>(grad, param, nullptr, v_row, R, C, beta2, c.eps1, ws));
  } else {
    T5MI_AF(af_norms_kernel, false><<<grid, 256, 0, st>>>(grad, param, v_full, nullptr, R, C, beta2, c.eps1, ws));
  }
  af_coef_kernel<<<1, 1024, 0, st>>>(g.ntiles, (double)R * (double)C, c, ws);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (factored)
    T5MI_AF(af_apply_kernel, true><<<grid, 256, 0, st>>>(param, grad, nullptr, v_row, (bf16*)bf16_out, R, C, ws));
  else
    T5MI_AF(af_apply_kernel, false><<<grid, 256, 0, st>>>(param, grad, v_full, nullptr, (bf16*)bf16_out, R, C, ws));
#undef T5MI_AF
  return hipSuccess;
}

}  // namespace t5mi
