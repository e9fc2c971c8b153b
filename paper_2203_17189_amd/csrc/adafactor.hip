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
//
// Every kernel works on a batch of up to 16 tensors at once (descriptor table passed by value, a
// workgroup finds its tensor from a prefix table of tile counts): a whole block's optimizer step is
// five launches, not five per tensor -- at T5.1.1-Base sizes the per-tensor launches cost more than
// the memory traffic.
#include "kernels.h"
#include <cmath>
#include <cstring>

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

struct AfItem {
  float* w;
  const float* g;
  float* v_row;
  float* v_col;
  float* v_full;
  bf16* lp;
  float* m;  // momentum (nullable)
  int64_t R, C;
  AfWs ws;
  int vec, ntc, ntr, factored;
};
struct AfBatch {
  AfItem it[AF_MAX_TENSORS];
  int tile_start[AF_MAX_TENSORS + 1];  // prefix sums of ntc * ntr
  int fin_start[AF_MAX_TENSORS + 1];   // prefix sums of ceil((R + C) / 256) over factored tensors
  int count;
  float beta2, eps1;
  float beta1, decay;  // momentum coefficient; lr * weight_decay
};

// Tensor that owns 1-D block `b` under prefix table `start` (wave-uniform).
__device__ __forceinline__ int af_find(const int* start, int count, int b) {
  int t = 0;
  while (t + 1 < count && b >= start[t + 1]) ++t;
  return t;
}

// Wave w takes rows w, w+4, ... of the tile; lanes span the columns.
template <int VEC>
__device__ __forceinline__ void af_stats_tile(const AfItem& it, int bx, int by, float (*colred)[256]) {
  const float* __restrict__ g = it.g;
  const int64_t R = it.R, C = it.C;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c0 = (int64_t)bx * 64 * VEC + lane * VEC;
  const int64_t r0 = (int64_t)by * TR;
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
    if (lane == 0) it.ws.rowpart[(int64_t)bx * R + r] = rs;
  }
#pragma unroll
  for (int i = 0; i < VEC; ++i) colred[wave][lane * VEC + i] = csum[i];
  __syncthreads();
  for (int t = threadIdx.x; t < 64 * VEC; t += 256) {
    const int64_t c = (int64_t)bx * 64 * VEC + t;
    if (c < C) it.ws.colpart[(int64_t)by * C + c] = colred[0][t] + colred[1][t] + colred[2][t] + colred[3][t];
  }
}

__global__ __launch_bounds__(256) void af_stats_kernel(AfBatch b) {
  __shared__ float colred[4][256];
  const int ti = af_find(b.tile_start, b.count, blockIdx.x);
  const AfItem& it = b.it[ti];
  if (!it.factored) return;
  const int local = blockIdx.x - b.tile_start[ti];
  const int bx = local % it.ntc, by = local / it.ntc;
  if (it.vec == 4) af_stats_tile<4>(it, bx, by, colred);
  else af_stats_tile<1>(it, bx, by, colred);
}

// One thread per row and per column: folds the tile partials into the second-moment vectors.
// cfac_j = rsqrt(v_col_j); the row factor needs mean(v_row) and is formed by the consumers.
__global__ __launch_bounds__(256) void af_finalize_kernel(AfBatch b) {
  const int ti = af_find(b.fin_start, b.count, blockIdx.x);
  const AfItem& it = b.it[ti];
  if (!it.factored) return;
  const int64_t R = it.R, C = it.C;
  const float beta2 = b.beta2, eps1 = b.eps1;
  const int64_t idx = (int64_t)(blockIdx.x - b.fin_start[ti]) * 256 + threadIdx.x;
  if (idx < R) {
    float s = 0.f;
    for (int t = 0; t < it.ntc; ++t) s += it.ws.rowpart[(int64_t)t * R + idx];
    it.v_row[idx] = beta2 * it.v_row[idx] + (1.f - beta2) * (s / (float)C + eps1);
  } else if (idx < R + C) {
    const int64_t j = idx - R;
    float s = 0.f;
    for (int t = 0; t < it.ntr; ++t) s += it.ws.colpart[(int64_t)t * C + j];
    const float vc = beta2 * it.v_col[j] + (1.f - beta2) * (s / (float)R + eps1);
    it.v_col[j] = vc;
    it.ws.cfac[j] = rsqrtf(vc);
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
__device__ __forceinline__ void af_norms_tile(const AfItem& it, int bx, int by, int tile, float beta2, float eps1,
                                              float* red) {
  const float* __restrict__ g = it.g;
  const float* __restrict__ w = it.w;
  float* __restrict__ v_full = it.v_full;
  const float* __restrict__ v_row = it.v_row;
  const int64_t R = it.R, C = it.C;
  const AfWs& ws = it.ws;
  float inv_mean = 1.f;
  if constexpr (FACT) {
    const float mean_vr = af_mean_vrow(v_row, R, red + 8);
    inv_mean = 1.f / mean_vr;
    if (tile == 0 && threadIdx.x == 0) ws.scal[1] = inv_mean;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c0 = (int64_t)bx * 64 * VEC + lane * VEC;
  const int64_t r0 = (int64_t)by * TR;
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
    ws.part_u[tile] = su;
    ws.part_w[tile] = sw;
  }
}

__global__ __launch_bounds__(256) void af_norms_kernel(AfBatch b) {
  __shared__ float red[12];
  const int ti = af_find(b.tile_start, b.count, blockIdx.x);
  const AfItem& it = b.it[ti];
  const int local = blockIdx.x - b.tile_start[ti];
  const int bx = local % it.ntc, by = local / it.ntc;
  if (it.vec == 4) {
    if (it.factored) af_norms_tile<4, true>(it, bx, by, local, b.beta2, b.eps1, red);
    else af_norms_tile<4, false>(it, bx, by, local, b.beta2, b.eps1, red);
  } else {
    if (it.factored) af_norms_tile<1, true>(it, bx, by, local, b.beta2, b.eps1, red);
    else af_norms_tile<1, false>(it, bx, by, local, b.beta2, b.eps1, red);
  }
}

// One workgroup per tensor.
__global__ __launch_bounds__(1024) void af_coef_kernel(AfBatch b, adafactor_cfg c) {
  __shared__ float red[32];
  const AfItem& it = b.it[blockIdx.x];
  const int64_t ntiles = (int64_t)it.ntc * it.ntr;
  float su = 0.f, sw = 0.f;
  for (int64_t i = threadIdx.x; i < ntiles; i += 1024) {
    su += it.ws.part_u[i];
    sw += it.ws.part_w[i];
  }
  su = block_sum<16>(su, red);
  sw = block_sum<16>(sw, red + 16);
  if (threadIdx.x == 0) {
    const double count = (double)it.R * (double)it.C;
    const float rms_u = sqrtf(su / (float)count), rms_w = sqrtf(sw / (float)count);
    float alpha = c.lr;
    if (c.scale_by_param) alpha *= fmaxf(c.eps2, rms_w);
    it.ws.scal[0] = alpha / fmaxf(1.f, rms_u / c.clip);
  }
}

// W <- W - D - decay W,  D = alpha U, or with momentum m <- beta1 m + (1 - beta1) alpha U, D = m
template <int VEC, bool FACT>
__device__ __forceinline__ void af_apply_tile(const AfItem& it, int bx, int by, float beta1, float decay) {
  float* __restrict__ w = it.w;
  const float* __restrict__ g = it.g;
  const float* __restrict__ v_full = it.v_full;
  const float* __restrict__ v_row = it.v_row;
  bf16* __restrict__ lp = it.lp;
  float* __restrict__ mom = it.m;
  const int64_t R = it.R, C = it.C;
  const AfWs& ws = it.ws;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t c0 = (int64_t)bx * 64 * VEC + lane * VEC;
  const int64_t r0 = (int64_t)by * TR;
  if (c0 >= C) return;
  const float coef = ws.scal[0];
  float cf[VEC];
  if constexpr (FACT) ldv<VEC>(ws.cfac + c0, cf);
  for (int rr = wave; rr < TR; rr += 4) {
    const int64_t r = r0 + rr;
    if (r >= R) break;
    float gv[VEC], wv[VEC], dv[VEC];
    ldv<VEC>(g + r * C + c0, gv);
    ldv<VEC>(w + r * C + c0, wv);
    if constexpr (FACT) {
      const float rf = rsqrtf(v_row[r] * ws.scal[1]) * coef;
#pragma unroll
      for (int i = 0; i < VEC; ++i) dv[i] = gv[i] * rf * cf[i];
    } else {
      float vv[VEC];
      ldv<VEC>(v_full + r * C + c0, vv);
#pragma unroll
      for (int i = 0; i < VEC; ++i) dv[i] = coef * gv[i] * rsqrtf(vv[i]);
    }
    if (mom) {
      float mv[VEC];
      ldv<VEC>(mom + r * C + c0, mv);
#pragma unroll
      for (int i = 0; i < VEC; ++i) { mv[i] = beta1 * mv[i] + (1.f - beta1) * dv[i]; dv[i] = mv[i]; }
      stv<VEC>(mom + r * C + c0, mv);
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) wv[i] = wv[i] - dv[i] - decay * wv[i];
    stv<VEC>(w + r * C + c0, wv);
    if (lp) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) lp[r * C + c0 + i] = (bf16)wv[i];
    }
  }
}

__global__ __launch_bounds__(256) void af_apply_kernel(AfBatch b) {
  const int ti = af_find(b.tile_start, b.count, blockIdx.x);
  const AfItem& it = b.it[ti];
  const int local = blockIdx.x - b.tile_start[ti];
  const int bx = local % it.ntc, by = local / it.ntc;
  if (it.vec == 4) {
    if (it.factored) af_apply_tile<4, true>(it, bx, by, b.beta1, b.decay);
    else af_apply_tile<4, false>(it, bx, by, b.beta1, b.decay);
  } else {
    if (it.factored) af_apply_tile<1, true>(it, bx, by, b.beta1, b.decay);
    else af_apply_tile<1, false>(it, bx, by, b.beta1, b.decay);
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

hipError_t launch_adafactor_multi(const AfTensor* t, int n, const adafactor_cfg& c, void* wsp, hipStream_t st) {
  if (n < 1 || n > AF_MAX_TENSORS) return hipErrorInvalidValue;
  AfBatch b;
  std::memset(&b, 0, sizeof(b));
  b.count = n;
  b.beta2 = (float)(1.0 - pow((double)c.step, -(double)c.decay_pow));
  b.eps1 = c.eps1;
  b.beta1 = c.beta1;
  b.decay = c.lr * c.weight_decay;
  char* wp = (char*)wsp;
  int64_t tiles = 0, fins = 0;
  bool any_factored = false;
  for (int i = 0; i < n; ++i) {
    const AfGeom g = geom(t[i].rows, t[i].cols);
    AfItem& it = b.it[i];
    it.w = t[i].param; it.g = t[i].grad; it.v_row = t[i].v_row; it.v_col = t[i].v_col; it.v_full = t[i].v_full;
    it.lp = (bf16*)t[i].bf16_out;
    it.m = c.beta1 > 0.f ? t[i].m : nullptr;
    it.R = t[i].rows; it.C = t[i].cols;
    it.ws = carve(wp, it.R, it.C, g);
    wp += adafactor_ws_bytes(it.R, it.C, t[i].factored);
    it.vec = g.vec; it.ntc = g.ntc; it.ntr = g.ntr; it.factored = t[i].factored ? 1 : 0;
    b.tile_start[i] = (int)tiles;
    b.fin_start[i] = (int)fins;
    tiles += g.ntiles;
    if (it.factored) { fins += ceil_div(it.R + it.C, (int64_t)256); any_factored = true; }
    if (tiles > (int64_t)1 << 30 || fins > (int64_t)1 << 30) return hipErrorInvalidValue;
  }
  for (int i = n; i <= AF_MAX_TENSORS; ++i) { b.tile_start[i] = (int)tiles; b.fin_start[i] = (int)fins; }
  hipError_t e;
  if (any_factored) {
    af_stats_kernel<<<(unsigned)tiles, 256, 0, st>>>(b);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    af_finalize_kernel<<<(unsigned)fins, 256, 0, st>>>(b);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  af_norms_kernel<<<(unsigned)tiles, 256, 0, st>>>(b);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  af_coef_kernel<<<n, 1024, 0, st>>>(b, c);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  af_apply_kernel<<<(unsigned)tiles, 256, 0, st>>>(b);
  return hipGetLastError();
}

hipError_t launch_adafactor(float* param, const float* grad, float* v_row, float* v_col, float* v_full,
                            int64_t R, int64_t C, int factored, const adafactor_cfg& c, void* bf16_out,
                            void* wsp, hipStream_t st) {
  AfTensor t{param, grad, v_row, v_col, v_full, R, C, factored, bf16_out, nullptr};
  return launch_adafactor_multi(&t, 1, c, wsp, st);
}

}  // namespace t5mi

// ------------------------------------------------------------------------------------------------
// adafactor_step_static: the single-tensor update for callers that cannot allocate.  Its scratch
// (the tile partial sums and factors that adafactor_step takes from the caller's workspace) is this
// file-scope device array; every GPU holds its own copy at its own address, looked up once per device.
// ------------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[ADAFACTOR_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU, set on first use there
}  // namespace

extern "C" int adafactor_step_static(float* param, const float* grad, float* v_row, float* v_col, float* v_full,
                                     int64_t rows, int64_t cols, int factored, const adafactor_cfg* cfg,
                                     void* bf16_copy_out, void* stream) {
  using namespace t5mi;
  if (!cfg) return T5_ERR_NULL;
  if (rows < 1 || cols < 1 || cfg->step < 1 || !(cfg->clip > 0.f) || !(cfg->eps1 >= 0.f)) return T5_ERR_SHAPE;
  if (!(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->weight_decay >= 0.f)) return T5_ERR_SHAPE;
  if (cfg->beta1 > 0.f) return T5_ERR_UNSUPPORTED;
  if (rows > (1 << 24) || cols > (1 << 24)) return T5_ERR_UNSUPPORTED;
  if (!param || !grad) return T5_ERR_NULL;
  if (factored ? (!v_row || !v_col) : !v_full) return T5_ERR_NULL;
  if (adafactor_ws_bytes(rows, cols, factored) > (size_t)ADAFACTOR_STATIC_SCRATCH_BYTES) return T5_ERR_WORKSPACE;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return T5_ERR_DEVICE;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return T5_ERR_DEVICE;
    g_scratch_ptr[dev] = p;
  }
  // Nothing in the scratch has to start at zero: every partial sum, factor and scalar a kernel of this
  // update reads was written by an earlier kernel of the same update.
  if (launch_adafactor(param, grad, v_row, v_col, v_full, rows, cols, factored, *cfg, bf16_copy_out,
                       g_scratch_ptr[dev], (hipStream_t)stream) != hipSuccess)
    return T5_ERR_DEVICE;
  return T5_OK;
}

