// Measurement aid: what the matrix units sustain on this machine with nothing else in the way.
// 256 threads per workgroup, one wave per SIMD, 16 independent 32x32 accumulators per wave, operands
// in registers; no LDS, no memory traffic.  With constant operands the chip holds its peak clock;
// with random bf16 operands it is power-limited and the clock drops, which is the ceiling a real
// GEMM lives under.
#include "kernels.h"

namespace t5mi {

namespace {

template <bool RANDOM>
__global__ __launch_bounds__(256, 1) void mfma_peak_kernel(float* sink, int iters) {
  f32x16 acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  bf16x8 av[4], bv[4];
  uint32_t h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
#pragma unroll
  for (int v = 0; v < 4; ++v)
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      h = h * 1664525u + 1013904223u;
      const float fa = RANDOM ? (float)((int)((h >> 8) % 2001u) - 1000) * 1e-3f : 1.f;
      h = h * 1664525u + 1013904223u;
      const float fb = RANDOM ? (float)((int)((h >> 8) % 2001u) - 1000) * 1e-3f : 1.f;
      av[v][q] = (bf16)fa;
      bv[v][q] = (bf16)fb;
    }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int rep = 0; rep < 2; ++rep)
#pragma unroll
      for (int i = 0; i < 16; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i & 3], bv[(i >> 2) & 3], acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  if (s == 12345.678f) sink[threadIdx.x] = s;  // keeps the loop alive; practically never taken
}

}  // namespace

hipError_t launch_mfma_peak_probe(int workgroups, int iters, int random_operands, float* sink, hipStream_t st) {
  if (random_operands) mfma_peak_kernel<true><<<workgroups, 256, 0, st>>>(sink, iters);
  else mfma_peak_kernel<false><<<workgroups, 256, 0, st>>>(sink, iters);
  return hipGetLastError();
}

}  // namespace t5mi
