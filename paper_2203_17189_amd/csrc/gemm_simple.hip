// Reference-grade GEMM for the float32 block and for bf16 shapes the MFMA kernel does not take:
// 64x64 output tile, 16-deep LDS stages, float32 FMA, any shape and either operand orientation.
// Also: the elementwise gated-GELU of the unfused path and the bf16 weight transpose-pack.
#include "kernels.h"
#include <algorithm>
#include <cstring>

namespace t5mi {

namespace {

constexpr int SB = 64;  // tile edge
constexpr int SK = 16;  // k depth per stage

__device__ __forceinline__ float ld_elem(const void* p, size_t idx, int type) {
  return type == IN_BF16 ? (float)((const bf16*)p)[idx] : ((const float*)p)[idx];
}
__device__ __forceinline__ void st_elem(void* p, size_t idx, int type, float v) {
  if (type == IN_BF16) ((bf16*)p)[idx] = (bf16)v; else ((float*)p)[idx] = v;
}

__global__ __launch_bounds__(256) void gemm_simple_kernel(GemmDesc g, GemmEpi e) {
  __shared__ float As[SK][SB + 1];
  __shared__ float Bs[SK][SB + 1];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  const int m0 = blockIdx.y * SB, n0 = blockIdx.x * SB;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int s = 0; s < g.nseg; ++s) {
    const GemmSeg sg = g.seg[s];
    for (int k0 = 0; k0 < sg.K; k0 += SK) {
      // 64x16 elements per operand, 256 threads -> 4 each
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int idx = tid + i * 256;
        int mm, kk;
        if (g.a_kc) { kk = idx % SK; mm = idx / SK; } else { mm = idx % SB; kk = idx / SB; }
        float v = 0.f;
        if (m0 + mm < g.M && k0 + kk < sg.K) {
          const size_t off = g.a_kc ? (size_t)(m0 + mm) * sg.lda + (k0 + kk)
                                    : (size_t)(k0 + kk) * sg.lda + (m0 + mm);
          v = ld_elem(sg.A, off, g.in_type);
        }
        As[kk][mm] = v;
        int nn, kb;
        if (g.b_kc) { kb = idx % SK; nn = idx / SK; } else { nn = idx % SB; kb = idx / SB; }
        float u = 0.f;
        if (n0 + nn < g.N && k0 + kb < sg.K) {
          const size_t off = g.b_kc ? (size_t)(n0 + nn) * sg.ldb + (k0 + kb)
                                    : (size_t)(k0 + kb) * sg.ldb + (n0 + nn);
          u = ld_elem(sg.B, off, g.in_type);
        }
        Bs[kb][nn] = u;
      }
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < SK; ++kk) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
      }
      __syncthreads();
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= g.N) continue;
      const float v = acc[i][j];
      const size_t o = (size_t)m * e.ld0 + n;
      const float mk = e.drop.on ? drop_mult(e.drop, drop_row_key(e.drop, (uint32_t)m), (uint32_t)n) : 1.f;
      switch (e.kind) {
        case EPI_STORE:
          st_elem(e.out0, o, e.out_type, (e.act == ACT_RELU ? fmaxf(v, 0.f) : v) * mk);
          break;
        case EPI_RESID: {
          const float a = ld_elem(e.aux0, (size_t)m * (e.ld_aux ? e.ld_aux : e.ld0) + n, e.aux_type);
          const float sc = e.drop.on ? e.drop.scale : 1.f;
          st_elem(e.out0, o, e.out_type, e.aux_mask ? (a > 0.f ? v * sc : 0.f) : v * mk + a);
          break;
        }
        case EPI_GEGLU_BWD: {
          const size_t oa = (size_t)m * (e.ld_aux ? e.ld_aux : e.ld0) + n;
          const float gp = ld_elem(e.aux0, oa, e.aux_type), gl = ld_elem(e.aux1, oa, e.aux_type);
          st_elem(e.out0, o, e.out_type, v * gp);
          st_elem(e.out1, o, e.out_type, v * gl);
          break;
        }
        case EPI_SPLIT_F32: {
          const int which = n / e.split_n, nn = n % e.split_n;
          float* dst = (float*)(which == 0 ? e.out0 : which == 1 ? e.out1 : e.out2);
          const size_t oo = (size_t)m * e.ld0 + nn;
          dst[oo] = e.accumulate ? dst[oo] + v : v;
          break;
        }
        default:
          break;
      }
    }
  }
}

template <typename T>
__global__ void geglu_fwd_kernel(T* __restrict__ u, T* __restrict__ w, T* __restrict__ a, int64_t n, int act,
                                 DropSite drop, int cols) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    const float uu = to_f32(u[i]), ww = to_f32(w[i]);
    float gl, dgl;
    gelu_both(act, uu, gl, dgl);
    // the saved factors carry the dropout multiplier of the hidden activation, for the backward
    const float mk = drop.on ? drop_mult(drop, drop_row_key(drop, (uint32_t)(i / cols)), (uint32_t)(i % cols)) : 1.f;
    a[i] = from_f32<T>(gl * ww * mk);
    u[i] = from_f32<T>(ww * dgl * mk);
    w[i] = from_f32<T>(gl * mk);
  }
}

// dst[n][k] for a 64x64 tile staged through LDS; see launch_pack_transpose_bf16.  blockIdx.z picks the
// job; blocks outside a job's tile range leave at once.  Each thread moves two adjacent elements, so
// a row of the tile is one 128-byte line on the way in and on the way out.
__global__ __launch_bounds__(256) void pack_transpose_kernel(PackJobs jobs) {
  __shared__ bf16 tile[64][66];
  const PackJob& jb = jobs.j[blockIdx.z];
  const int nsrc = jb.nsrc, K = jb.K, n_each = jb.n_each, interleave = jb.interleave;
  const int n_total = nsrc * n_each;
  const int n0 = blockIdx.x * 64, k0 = blockIdx.y * 64;
  if (n0 >= n_total || k0 >= K) return;
  const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;  // 32 column pairs x 8 rows
  // interleave and n_each are multiples of 32 (or interleave == 0), so each 32-wide half of the tile's packed
  // rows comes from one source and 32 consecutive source columns; a thread's pair lies inside one half.
  const int c = 2 * tx, nh = n0 + (c & 32);  // first packed row of this thread's half
  int which, col0;
  if (interleave > 0) {
    which = (nh / interleave) % nsrc;
    col0 = (nh / (interleave * nsrc)) * interleave + nh % interleave;
  } else {
    which = nh / n_each;
    col0 = nh % n_each;
  }
  const bool in_n = nh < n_total;
  const bf16* src = (const bf16*)jb.src[in_n ? which : 0];
  bf16* dst = (bf16*)jb.dst;
  for (int r = ty; r < 64; r += 8) {
    const int k = k0 + r;
    uint32_t v = 0;
    if (in_n && k < K) v = *reinterpret_cast<const uint32_t*>(src + (size_t)k * n_each + col0 + (c & 31));
    *reinterpret_cast<uint32_t*>(&tile[r][c]) = v;
  }
  __syncthreads();
  for (int r = ty; r < 64; r += 8) {
    const int n = n0 + r, k = k0 + c;
    if (n < n_total && k < K) {  // K is even: the pair (k, k + 1) is inside or outside together
      const uint32_t lo = __builtin_bit_cast(uint16_t, tile[c][r]), hi = __builtin_bit_cast(uint16_t, tile[c + 1][r]);
      *reinterpret_cast<uint32_t*>(dst + (size_t)n * K + k) = lo | (hi << 16);
    }
  }
}

}  // namespace

hipError_t launch_gemm_simple(const GemmDesc& g, const GemmEpi& e, hipStream_t st) {
  if (e.kind == EPI_GEGLU_FWD) return hipErrorInvalidValue;
  dim3 grid(ceil_div(g.N, SB), ceil_div(g.M, SB));
  gemm_simple_kernel<<<grid, 256, 0, st>>>(g, e);
  return hipGetLastError();
}

__global__ void zero_f32_kernel(ZeroList z) {
  const int a = blockIdx.y;
  float* p = z.p[a];
  const int64_t n = z.n[a];
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    p[i] = 0.f;
}

hipError_t launch_zero_f32(const ZeroList& z, hipStream_t st) {
  if (z.count <= 0) return hipSuccess;
  int64_t mx = 0;
  for (int a = 0; a < z.count; ++a) mx = z.n[a] > mx ? z.n[a] : mx;
  const int64_t blocks = std::min<int64_t>((mx + 255) / 256, 1024);
  zero_f32_kernel<<<dim3((unsigned)std::max<int64_t>(blocks, 1), (unsigned)z.count), 256, 0, st>>>(z);
  return hipGetLastError();
}

hipError_t launch_geglu_fwd(void* u, void* w, void* a, int type, int64_t n, int act, const DropSite& drop, int cols,
                            hipStream_t st) {
  int64_t blocks = (n + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  if (type == IN_BF16)
    geglu_fwd_kernel<bf16><<<(int)blocks, 256, 0, st>>>((bf16*)u, (bf16*)w, (bf16*)a, n, act, drop, cols);
  else
    geglu_fwd_kernel<float><<<(int)blocks, 256, 0, st>>>((float*)u, (float*)w, (float*)a, n, act, drop, cols);
  return hipGetLastError();
}

hipError_t launch_pack_transpose_multi(const PackJobs& jobs, hipStream_t st) {
  if (jobs.count < 1 || jobs.count > 8) return hipErrorInvalidValue;
  int gx = 0, gy = 0;
  for (int q = 0; q < jobs.count; ++q) {
    const PackJob& jb = jobs.j[q];
    if (jb.nsrc < 1 || jb.nsrc > 3 || jb.n_each % 32 != 0 || (jb.interleave > 0 && jb.interleave % 32 != 0) ||
        jb.K % 2 != 0)
      return hipErrorInvalidValue;
    gx = std::max(gx, ceil_div(jb.nsrc * jb.n_each, 64));
    gy = std::max(gy, ceil_div(jb.K, 64));
  }
  pack_transpose_kernel<<<dim3(gx, gy, jobs.count), 256, 0, st>>>(jobs);
  return hipGetLastError();
}

hipError_t launch_pack_transpose_bf16(const void* const* srcs, int nsrc, int K, int n_each, void* dst,
                                      int interleave, hipStream_t st) {
  if (nsrc < 1 || nsrc > 3) return hipErrorInvalidValue;
  PackJobs jobs;
  std::memset(&jobs, 0, sizeof(jobs));
  for (int i = 0; i < nsrc; ++i) jobs.j[0].src[i] = srcs[i];
  jobs.j[0].nsrc = nsrc; jobs.j[0].K = K; jobs.j[0].n_each = n_each; jobs.j[0].interleave = interleave;
  jobs.j[0].dst = dst;
  jobs.count = 1;
  return launch_pack_transpose_multi(jobs, st);
}

}  // namespace t5mi
