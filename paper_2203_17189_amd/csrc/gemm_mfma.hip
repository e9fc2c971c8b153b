// bf16 MFMA GEMM for gfx950 (v_mfma_f32_32x32x16_bf16, float32 accumulation) with fused epilogues.
//
//   C[m,n] = sum_s sum_k A_s(m,k) B_s(n,k)
//
// Tiling: workgroup tile BM x BN x 64, WM x WN wavefronts, each wave owns (BM/WM) x (BN/WN) as
// 32x32 MFMA tiles.  Operand tiles go global -> registers -> LDS (double buffered, one barrier per
// k-tile).  Two LDS layouts:
//   k-contiguous operand (A[m][k]):  rows of 64 k (128 B), 16-byte chunks XOR-swizzled by row, read
//                                    with ds_read_b128;
//   m-contiguous operand (A[k][m]):  rows of BM m, 32-byte granules XOR-swizzled by k, read with the
//                                    LDS transpose load ds_read_b64_tr_b16 (two per MFMA operand).
// Workgroup ids are remapped so that each XCD (ids are dealt round-robin to the 8 XCDs) works on a
// compact block of output tiles and shares operand tiles through its own L2.
#include "kernels.h"

namespace t5mi {

namespace {

constexpr int BK = 64;

typedef __attribute__((address_space(3))) short4v lds_short4;

__device__ __forceinline__ int swz_row(int row) { return (row ^ (row >> 3)) & 7; }

template <int ROWS, bool KC>
struct TileLds {
  // byte offset of the 16-byte chunk `chunk` of row `row` (KC: row = m, chunk = k/8;
  // !KC: row = k, chunk = m/8) inside one stage
  __device__ static __forceinline__ int chunk_off(int row, int chunk) {
    if constexpr (KC) {
      return row * 128 + ((chunk ^ swz_row(row)) << 4);
    } else {
      const int g = chunk >> 1, half = chunk & 1;
      return row * (ROWS * 2) + (((g ^ ((row & 3) << 1))) << 5) + (half << 4);
    }
  }
};

// One MFMA operand (8 bf16 of k for row `mrow` = base + lane%32) for k-step kk of the stage.
template <int ROWS, bool KC>
__device__ __forceinline__ bf16x8 load_frag(const char* stage, int base, int kk, int lane) {
  if constexpr (KC) {
    const int row = base + (lane & 31);
    const int chunk = kk * 2 + (lane >> 5);
    return *reinterpret_cast<const bf16x8*>(stage + TileLds<ROWS, true>::chunk_off(row, chunk));
  } else {
    // 16-lane groups: lanes supply the address of 4 consecutive m at row k; the transpose load hands
    // lane i the 4 k-values of m = group_base + i.
    const int i16 = lane & 15;
    const int m_e = base + (((lane >> 4) & 1) << 4) + ((i16 & 3) << 2);
    const int krow = kk * 16 + ((lane >> 5) << 3) + (i16 >> 2);
    const int g = m_e >> 4;
    const int off0 = krow * (ROWS * 2) + ((g ^ ((krow & 3) << 1)) << 5) + ((m_e & 15) << 1);
    const int off1 = off0 + 4 * (ROWS * 2);  // krow + 4 keeps (krow & 3)
    short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(stage + off0));
    short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(stage + off1));
    typedef __attribute__((ext_vector_type(8))) short short8v;
    short8v r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, r);
  }
}

struct KTile {
  const bf16* a;
  const bf16* b;
  int lda, ldb, k0;
};

template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(WM * WN * 64) void gemm_mfma_kernel(GemmDesc g, GemmEpi e, int tiles_m,
                                                                int tiles_n, int split_k) {
  constexpr int NT = WM * WN * 64;
  constexpr int TMW = BM / WM, TNW = BN / WN;
  constexpr int MI = TMW / 32, NI = TNW / 32;
  constexpr int A_CH = BM * 8 / NT, B_CH = BN * 8 / NT;  // 16-byte chunks per thread per k-tile
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128;
  constexpr int STAGE = A_BYTES + B_BYTES;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // ---- XCD-aware tile mapping
  const int nb = tiles_m * tiles_n;
  int bid = blockIdx.x;
  const int ks = bid / nb;  // split-k slice
  bid -= ks * nb;
  int L;
  {
    const int xcd = bid & 7, idx = bid >> 3;
    const int nb8 = (nb + 7) >> 3, rem = nb & 7;
    if (rem == 0 || xcd < rem) L = xcd * nb8 + idx; else L = rem * nb8 + (xcd - rem) * (nb8 - 1) + idx;
  }
  constexpr int GM = 8;
  const int per_group = GM * tiles_n;
  const int group = L / per_group, in_g = L - group * per_group;
  const int first_m = group * GM;
  const int gsz = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
  const int tm = first_m + in_g % gsz, tn = in_g / gsz;
  const int m0 = tm * BM, n0 = tn * BN;

  // ---- k-tile range of this workgroup (flattened over segments)
  int nk_total = 0;
  for (int s = 0; s < g.nseg; ++s) nk_total += g.seg[s].K / BK;
  const int per = (nk_total + split_k - 1) / split_k;
  const int kt_begin = ks * per;
  const int kt_end = (kt_begin + per) < nk_total ? (kt_begin + per) : nk_total;

  auto tile_at = [&](int kt) {
    KTile t;
    int s = 0, base = 0;
    while (s + 1 < g.nseg && kt >= base + g.seg[s].K / BK) { base += g.seg[s].K / BK; ++s; }
    t.a = (const bf16*)g.seg[s].A;
    t.b = (const bf16*)g.seg[s].B;
    t.lda = g.seg[s].lda;
    t.ldb = g.seg[s].ldb;
    t.k0 = (kt - base) * BK;
    return t;
  };

  u32x4 areg[A_CH], breg[B_CH];
  auto gload = [&](int kt) {
    const KTile t = tile_at(kt);
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int q = tid + i * NT;
      const bf16* p;
      if constexpr (A_KC) {
        int row = m0 + (q >> 3);
        row = row < g.M ? row : g.M - 1;
        p = t.a + (size_t)row * t.lda + t.k0 + ((q & 7) << 3);
      } else {
        const int krow = q / (BM / 8), cm = q % (BM / 8);
        int mm = m0 + cm * 8;
        mm = mm < g.M ? mm : g.M - 8;
        p = t.a + (size_t)(t.k0 + krow) * t.lda + mm;
      }
      areg[i] = *reinterpret_cast<const u32x4*>(p);
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
      const int q = tid + i * NT;
      const bf16* p;
      if constexpr (B_KC) {
        int row = n0 + (q >> 3);
        row = row < g.N ? row : g.N - 1;
        p = t.b + (size_t)row * t.ldb + t.k0 + ((q & 7) << 3);
      } else {
        const int krow = q / (BN / 8), cn = q % (BN / 8);
        int nn = n0 + cn * 8;
        nn = nn < g.N ? nn : g.N - 8;
        p = t.b + (size_t)(t.k0 + krow) * t.ldb + nn;
      }
      breg[i] = *reinterpret_cast<const u32x4*>(p);
    }
  };
  auto lstore = [&](int buf) {
    char* sa = smem + buf * STAGE;
    char* sb = sa + A_BYTES;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int q = tid + i * NT;
      int off;
      if constexpr (A_KC) off = TileLds<BM, true>::chunk_off(q >> 3, q & 7);
      else off = TileLds<BM, false>::chunk_off(q / (BM / 8), q % (BM / 8));
      *reinterpret_cast<u32x4*>(sa + off) = areg[i];
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
      const int q = tid + i * NT;
      int off;
      if constexpr (B_KC) off = TileLds<BN, true>::chunk_off(q >> 3, q & 7);
      else off = TileLds<BN, false>::chunk_off(q / (BN / 8), q % (BN / 8));
      *reinterpret_cast<u32x4*>(sb + off) = breg[i];
    }
  };

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  if (kt_begin < kt_end) {
    gload(kt_begin);
    lstore(0);
    __syncthreads();
    for (int kt = kt_begin; kt < kt_end; ++kt) {
      const int buf = (kt - kt_begin) & 1;
      const bool more = kt + 1 < kt_end;
      if (more) gload(kt + 1);
      const char* sa = smem + buf * STAGE;
      const char* sb = sa + A_BYTES;
#pragma unroll
      for (int kk = 0; kk < BK / 16; ++kk) {
        bf16x8 af[MI], bfr[NI];
#pragma unroll
        for (int i = 0; i < MI; ++i) af[i] = load_frag<BM, A_KC>(sa, wm * TMW + i * 32, kk, lane);
#pragma unroll
        for (int j = 0; j < NI; ++j) bfr[j] = load_frag<BN, B_KC>(sb, wn * TNW + j * 32, kk, lane);
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < NI; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
      }
      if (more) lstore(buf ^ 1);
      __syncthreads();
    }
  }

  // ---- epilogue.  acc[i][j][r]: row = (r/4)*8 + (lane/32)*4 + r%4, col = lane%32 of the 32x32 tile.
  const int col_l = lane & 31, row_l = (lane >> 5) << 2;
#pragma unroll
  for (int i = 0; i < MI; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int m = m0 + wm * TMW + i * 32 + ((r >> 2) << 3) + row_l + (r & 3);
      if (m >= g.M) continue;
      if constexpr (EPI == EPI_GEGLU_FWD) {
#pragma unroll
        for (int j = 0; j < NI; j += 2) {
          const int n = n0 + wn * TNW + j * 32;  // packed column of the u tile; w tile follows
          if (n >= g.N) continue;
          const int f = (n >> 6) * 32 + col_l;
          // round u and w to storage precision first so the saved values reproduce `a` in the backward
          const bf16 ub = (bf16)acc[i][j][r], wb = (bf16)acc[i][j + 1][r];
          const size_t o = (size_t)m * e.ld0 + f;
          ((bf16*)e.out0)[o] = ub;
          ((bf16*)e.out1)[o] = wb;
          ((bf16*)e.out2)[o] = (bf16)(gelu_tanh((float)ub) * (float)wb);
        }
      } else {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
          const int n = n0 + wn * TNW + j * 32 + col_l;
          if (n >= g.N) continue;
          const float v = acc[i][j][r];
          const size_t o = (size_t)m * e.ld0 + n;
          if constexpr (EPI == EPI_STORE) {
            if (e.out_type == IN_BF16) ((bf16*)e.out0)[o] = (bf16)v; else ((float*)e.out0)[o] = v;
          } else if constexpr (EPI == EPI_RESID) {
            const float a = e.aux_type == IN_BF16 ? (float)((const bf16*)e.aux0)[o] : ((const float*)e.aux0)[o];
            if (e.out_type == IN_BF16) ((bf16*)e.out0)[o] = (bf16)(v + a); else ((float*)e.out0)[o] = v + a;
          } else if constexpr (EPI == EPI_GEGLU_BWD) {
            const float u = (float)((const bf16*)e.aux0)[o], w = (float)((const bf16*)e.aux1)[o];
            float gl, dgl;
            gelu_tanh_both(u, gl, dgl);
            ((bf16*)e.out0)[o] = (bf16)(v * w * dgl);
            ((bf16*)e.out1)[o] = (bf16)(v * gl);
          } else {  // EPI_SPLIT_F32
            const int which = n / e.split_n, nn = n - which * e.split_n;
            float* dst = (float*)(which == 0 ? e.out0 : which == 1 ? e.out1 : e.out2) + (size_t)m * e.ld0 + nn;
            if (split_k > 1) unsafeAtomicAdd(dst, v);
            else *dst = e.accumulate ? *dst + v : v;
          }
        }
      }
    }
  }
}

__global__ void zero_split_kernel(GemmEpi e, int M, int N) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)M * N) return;
  const int m = (int)(idx / N), n = (int)(idx % N);
  const int which = n / e.split_n, nn = n - which * e.split_n;
  float* dst = (float*)(which == 0 ? e.out0 : which == 1 ? e.out1 : e.out2);
  dst[(size_t)m * e.ld0 + nn] = 0.f;
}

template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, int EPI>
hipError_t launch_cfg(const GemmDesc& g, const GemmEpi& e, int split_k, hipStream_t st) {
  auto kern = gemm_mfma_kernel<BM, BN, WM, WN, A_KC, B_KC, EPI>;
  constexpr int lds = 2 * (BM + BN) * 128;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (err != hipSuccess) return err;
    attr_set = true;
  }
  const int tiles_m = ceil_div(g.M, BM), tiles_n = ceil_div(g.N, BN);
  kern<<<tiles_m * tiles_n * split_k, WM * WN * 64, lds, st>>>(g, e, tiles_m, tiles_n, split_k);
  return hipGetLastError();
}

template <bool A_KC, bool B_KC, int EPI>
hipError_t launch_layout(const GemmDesc& g, const GemmEpi& e, hipStream_t st) {
  int nk = 0;
  for (int s = 0; s < g.nseg; ++s) nk += g.seg[s].K / BK;
  const int64_t big_tiles = (int64_t)ceil_div(g.M, 256) * ceil_div(g.N, 256);
  const bool big = big_tiles >= 192 || EPI == EPI_SPLIT_F32;
  int split_k = 1;
  if constexpr (EPI == EPI_SPLIT_F32) {
    // weight-gradient GEMMs: few output tiles, very long k.  Split k so about two workgroups per
    // compute unit exist; partial sums meet in float32 atomics on a zeroed output.
    while (big_tiles * split_k < 384 && nk / (split_k * 2) >= 8) split_k *= 2;
    if (split_k > 1 && !e.accumulate) {
      zero_split_kernel<<<ceil_div((int64_t)g.M * g.N, 256), 256, 0, st>>>(e, g.M, g.N);
      hipError_t err = hipGetLastError();
      if (err != hipSuccess) return err;
    }
  }
  if (big) return launch_cfg<256, 256, 2, 2, A_KC, B_KC, EPI>(g, e, split_k, st);
  return launch_cfg<128, 128, 2, 2, A_KC, B_KC, EPI>(g, e, split_k, st);
}

}  // namespace

bool gemm_mfma_supported(const GemmDesc& g, const GemmEpi& e) {
  if (g.in_type != IN_BF16) return false;
  if (g.nseg < 1 || g.nseg > 3) return false;
  if (g.a_kc != g.b_kc) return false;  // implemented: both k-contiguous, or both m/n-contiguous
  for (int s = 0; s < g.nseg; ++s) {
    const GemmSeg& sg = g.seg[s];
    if (sg.K < BK || sg.K % BK != 0 || sg.lda % 8 != 0 || sg.ldb % 8 != 0) return false;
    if (((uintptr_t)sg.A | (uintptr_t)sg.B) & 15) return false;
  }
  if (g.M < 8 || g.N < 8) return false;
  if (!g.a_kc && (g.M % 8 != 0 || g.N % 8 != 0)) return false;
  switch (e.kind) {
    case EPI_STORE: case EPI_RESID: case EPI_GEGLU_BWD:
      return g.a_kc == 1;
    case EPI_GEGLU_FWD:
      return g.a_kc == 1 && g.N % 64 == 0 && e.out_type == IN_BF16;
    case EPI_SPLIT_F32:
      return g.a_kc == 0;
    default:
      return false;
  }
}

hipError_t launch_gemm_mfma(const GemmDesc& g, const GemmEpi& e, hipStream_t st) {
  switch (e.kind) {
    case EPI_STORE: return launch_layout<true, true, EPI_STORE>(g, e, st);
    case EPI_RESID: return launch_layout<true, true, EPI_RESID>(g, e, st);
    case EPI_GEGLU_FWD: return launch_layout<true, true, EPI_GEGLU_FWD>(g, e, st);
    case EPI_GEGLU_BWD: return launch_layout<true, true, EPI_GEGLU_BWD>(g, e, st);
    case EPI_SPLIT_F32: return launch_layout<false, false, EPI_SPLIT_F32>(g, e, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace t5mi
