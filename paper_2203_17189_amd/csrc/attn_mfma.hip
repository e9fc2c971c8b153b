// Fused attention for gfx950 (bf16 MFMA 32x32x16, float32 online softmax): self-attention with the
// T5 relative-position bias (BIAS, optionally CAUSAL), or cross-attention of S queries over Sk keys
// of another sequence without bias or mask.  The S x Sk scores never leave registers.
//
// Forward and the dq kernel give each lane one query: scores are computed transposed,
// S^T = K Q^T, so the MFMA result layout puts a query in lane%32 and 16 keys of a 32-key tile in
// the lane's registers.  Row maxima and sums are then register reductions plus one exchange between
// the two lane halves, and the probabilities feed the second matmul (O^T = V^T P^T) straight from
// the result registers: the contraction index of an MFMA may be permuted freely as long as both
// operands use the same permutation, and the V^T operand is fetched with that permutation by the
// LDS transpose load.  The dk/dv kernel mirrors this with one key per lane (S = Q K^T).
//
// Dropout of the probabilities (DROP): the keep decision of element
// ((b*H + h)*S + i, j) is regenerated from the counter-based generator where P is formed -- the lane
// that owns a query (forward, dq) hashes its row key once, the dk/dv kernel stages the row keys of a
// query tile in LDS beside -lse and -dvec.  The factor 1/(1 - rate) of the kept probabilities is applied
// to the finished O and dV accumulators, and to dP before dvec is subtracted.
//
// Sequence lengths need not be multiples of the tile sizes: tiles are rounded up, rows past the end are
// fetched from the last valid row, keys past the end are masked like causal ones, and queries past the end
// are neither stored nor counted in the bias gradient.
//
// The bias is Toeplitz: bias[h,i,j] = diag[h][j - i + S - 1].  Each workgroup stages the slice of
// the per-head diagonal vector it can touch (S + tile - 1 floats) in LDS.
#include "kernels.h"

namespace t5mi {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef __attribute__((address_space(3))) short4v lds_short4;
typedef __attribute__((ext_vector_type(8))) short short8v;

// Row-dependent XOR applied to the 16-byte chunk index of a [rows][DK] bf16 tile.  Chosen so that
// both access patterns are bank-conflict free: 16 consecutive rows x one chunk (ds_read_b128
// operand reads) and 4 consecutive rows x 4 consecutive chunks (transpose reads).
template <int DK>
__device__ __forceinline__ int row_swz(int row) {
  if constexpr (DK == 64)
    return (((row >> 1) & 1) << 2) | (((row >> 2) & 1) << 1) | ((row >> 3) & 1);
  else
    return ((row & 1) << 2) | (((row >> 1) & 1) << 3) | ((row >> 2) & 1) | (((row >> 3) & 1) << 1);
}
template <int DK>
__device__ __forceinline__ int tile_off(int row, int chunk) {
  return row * (DK * 2) + ((chunk ^ row_swz<DK>(row)) << 4);
}

// Cooperative copy of `rows` rows of DK bf16 (row r at src + r*ld) into a swizzled LDS tile.
// Rows at or beyond `valid` are clamped to the last valid row (their results are never used).
template <int DK, int NT>
__device__ __forceinline__ void load_tile(char* dst, const bf16* __restrict__ src, size_t ld, int rows,
                                          int valid, int tid) {
  constexpr int CPR = DK / 8;
  for (int q = tid; q < rows * CPR; q += NT) {
    const int row = q / CPR, ch = q % CPR;
    const int rs = row < valid ? row : valid - 1;
    *reinterpret_cast<u32x4*>(dst + tile_off<DK>(row, ch)) =
        *reinterpret_cast<const u32x4*>(src + (size_t)rs * ld + ch * 8);
  }
}

// DMA descriptor of one [ROWS][DK] bf16 tile for a 4-wave workgroup: the tile is ROWS*DK*2/1024
// blocks of 1 KB, wave w copies blocks w, w+4, ...  The swizzle of tile_off() is applied on the
// global side: the lane that owns LDS slot (row, physical chunk) fetches the logical chunk.
template <int DK, int ROWS>
struct TileDma {
  static constexpr int PER_WAVE = ROWS * DK * 2 / 1024 / 4;
  uint32_t voff[PER_WAVE];
  // valid: rows of the tile that exist; the others fetch the last valid row again (their values are masked
  // or never stored), so that a ragged last tile reads nothing outside the operand
  __device__ __forceinline__ void init(int wave, int lane, size_t ld_elems, int valid = ROWS) {
    constexpr int CPR = DK / 8;
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
      const int slot = (wave + i * 4) * 64 + lane;
      const int row = slot / CPR, pch = slot % CPR;
      const int src = row < valid ? row : valid - 1;
      voff[i] = (uint32_t)(src * ld_elems * 2) + (uint32_t)((pch ^ row_swz<DK>(row)) << 4);
    }
  }
  __device__ __forceinline__ void issue(uint32_t lds_addr, const void* sbase, int wave) const {
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) dma_1k(lds_addr + (wave + i * 4) * 1024, sbase, voff[i]);
  }
};

// All DMA issued so far has landed, this wave's LDS traffic is complete, and every wave is here.
// 64 floats global -> LDS, one per lane (global_load_lds_dword): lane L fetches 4 bytes at sbase + voff and they
// land at LDS address lds_addr + 4*L.  Same ordering rules as the 1 KB form.
__device__ __forceinline__ void dma_64f(uint32_t lds_addr, const void* sbase, uint32_t voff) {
  lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_addr), "v"(voff), "s"(sbase));
}

__device__ __forceinline__ void dma_wait_barrier() {
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Operand with 8 consecutive channels of row (base + lane%32): k-step kk covers channels kk*16..+15.
template <int DK>
__device__ __forceinline__ bf16x8 frag_rows(const char* tile, int base, int kk, int lane) {
  return *reinterpret_cast<const bf16x8*>(tile + tile_off<DK>(base + (lane & 31), kk * 2 + (lane >> 5)));
}

// Transposed operand: MFMA row = channel (cbase + lane%32), contraction over tile rows.  Slot jj of
// lane half g holds tile row  rbase + 8*(jj/4) + 4*g + jj%4  -- the order in which the 32x32 result
// layout keeps rows 8*(r/4) + 4*g + r%4 in consecutive registers.
template <int DK>
__device__ __forceinline__ bf16x8 frag_cols_tr(const char* tile, int rbase, int cbase, int lane) {
  const int i16 = lane & 15;
  const int ch_e = cbase + (((lane >> 4) & 1) << 4) + ((i16 & 3) << 2);  // first of 4 channels addressed
  const int row0 = rbase + ((lane >> 5) << 2) + (i16 >> 2);
  const int row1 = row0 + 8;
  const int o0 = tile_off<DK>(row0, ch_e >> 3) + ((ch_e & 7) << 1);
  const int o1 = tile_off<DK>(row1, ch_e >> 3) + ((ch_e & 7) << 1);
  short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(tile + o0));
  short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(tile + o1));
  short8v r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, r);
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int first) {
  bf16x8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = (bf16)v[first + i];
  return o;
}

// Workgroup -> (tile, head, batch).  Workgroup ids are dealt round-robin to the 8 XCDs; the tiles of
// one (batch, head) share its K/V (or Q/dO) stream, so they are given ids that are congruent mod 8
// and adjacent in dispatch order: they run on one XCD at about the same time and share its L2.
__device__ __forceinline__ void decode_block(int n_tiles, int H, int B, int& tile, int& h, int& b) {
  const int bh_total = H * B;
  const int id = blockIdx.x;
  int bh;
  if ((bh_total & 7) == 0) {
    const int xcd = id & 7, j = id >> 3;
    bh = (j / n_tiles) * 8 + xcd;
    tile = j % n_tiles;
  } else {
    bh = id / n_tiles;
    tile = id % n_tiles;
  }
  h = bh % H;
  b = bh / H;
}

// dg[t] = src[idx_of(t)] * log2(e) for t in [0, n): 256 threads, four independent loads in flight per
// thread (the slice is short, so its load latency is all there is to hide).
template <typename F>
__device__ __forceinline__ void fill_bias_slice(float* dg, const float* __restrict__ src, int n, int tid, F idx_of) {
  for (int t0 = tid; t0 < n; t0 += 4 * 256) {
    float v[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int t = t0 + q * 256;
      v[q] = src[idx_of(t < n ? t : n - 1)];
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int t = t0 + q * 256;
      if (t < n) dg[t] = v[q] * kLog2e;
    }
  }
}

// Registers R.. of a 32x32 ds sub-tile (S^T layout), each rotated across the 32 lanes of its half by
// its key offset, summed into `tot`; `lo` gets the part whose source query did not wrap around
// (lp = 31 - query index of the receiving lane).  The rotation amount must be an immediate.
// The rotations are issued in groups of eight before any of their results is used: one at a time, each
// is followed by a wait for its trip through the LDS crossbar.
template <int R>
__device__ __forceinline__ float diag_rot(const f32x16& ds) {
  constexpr int kj0 = ((R >> 2) << 3) + (R & 3);  // key offset of register R (without the half's + 4)
  const float x = ds[R];  // (a plain float first: bit-casting the vector element itself picks element 0)
  return __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, x), 0xC000 | (kj0 << 5)));
}
template <int R0>
__device__ __forceinline__ void diag_accum8(const f32x16& ds, int lp, float& lo, float& tot) {
  const float v0 = diag_rot<R0>(ds), v1 = diag_rot<R0 + 1>(ds), v2 = diag_rot<R0 + 2>(ds), v3 = diag_rot<R0 + 3>(ds);
  const float v4 = diag_rot<R0 + 4>(ds), v5 = diag_rot<R0 + 5>(ds), v6 = diag_rot<R0 + 6>(ds), v7 = diag_rot<R0 + 7>(ds);
  __builtin_amdgcn_sched_barrier(0);
  const float v[8] = {v0, v1, v2, v3, v4, v5, v6, v7};
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int r = R0 + q;
    const int kj0 = ((r >> 2) << 3) + (r & 3);
    lo += lp >= kj0 ? v[q] : 0.f;
    tot += v[q];
  }
}
__device__ __forceinline__ void diag_accum(const f32x16& ds, int lp, float& lo, float& tot) {
  diag_accum8<0>(ds, lp, lo, tot);
  diag_accum8<8>(ds, lp, lo, tot);
}

// Number of 32-key blocks on each side of a wave's queries whose diagonals are resolved one by one in
// the dq kernel: offsets up to far + 30 can fall into a sub-tile that is not entirely saturated.
__host__ __device__ inline int attn_dq_window_blocks(int S, int far) {
  const int nb = (far + 30) / 32, cap = (S + 31) / 32 - 1;
  return nb < cap ? nb : cap;
}
// Floats per workgroup row of the reproducible bias-gradient buffer: a window is at most 64 * ceil(S / 32)
// entries wide (+ 4 for the upper lane half) and two sums of the saturated buckets follow it.
__host__ __device__ inline int attn_ddiag_part_stride(int S) { return 64 * ((S + 31) / 32) + 8; }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// max(x of this lane, x of the lane 32 away).  v_permlane32_swap exchanges lanes 32..63 of its first operand with
// lanes 0..31 of its second: started from two copies of x, every lane then holds its own value in one of the two
// registers and its partner's in the other.  One vector instruction through no memory, where the generic shuffle
// is an LDS round trip (ds_bpermute) on the dependent chain of every key tile.  (The s_nop covers the wait states
// between a vector write of the operands and the swap; the compiler's builtin for this instruction returned the
// same half in both results when tried here, hence the assembly.)
__device__ __forceinline__ float max_across_halves(float x) {
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  return fmaxf(a, b);
}

// ------------------------------------------------------------------------------------------------
// Forward.  grid (ceil(S/128), H, B), 256 threads; wave w owns queries i0 + 32w + lane%32.
// ------------------------------------------------------------------------------------------------
template <int DK, bool CAUSAL, bool BIAS, bool DROP>
__global__ __launch_bounds__(256, 2) void attn_fwd_mfma_kernel(AttnIO io, const float* __restrict__ diag,
                                                            bf16* __restrict__ c, float* __restrict__ lse,
                                                            AttnDims a) {
  constexpr int BR = 128, BC = 64, KS = DK / 16, CT = DK / 32;
  constexpr int TILE = BC * DK * 2, STG = 2 * TILE;  // a stage holds a K tile then a V tile
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  float* dg = reinterpret_cast<float*>(smem + 2 * STG);  // [S + BR - 1], log2 units (BIAS only)

  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int S = a.S, Sk = a.Sk, I = a.H * DK;
  const size_t ldq = (size_t)io.ldq, ld = (size_t)io.ldkv;
  int qt, h, b;
  decode_block((S + BR - 1) / BR, a.H, a.B, qt, h, b);
  if (CAUSAL) qt = (S + BR - 1) / BR - 1 - qt;  // heavy causal tiles first
  const int i0 = qt * BR;
  const int i_loc = wave * 32 + (lane & 31);
  const int i = i0 + i_loc;
  const int i_ld = i < S ? i : S - 1;
  const bf16* kbase = (const bf16*)io.k + (size_t)b * Sk * ld + h * DK;
  const bf16* vbase = (const bf16*)io.v + (size_t)b * Sk * ld + h * DK;

  bf16x8 qf[KS];
  {
    const bf16* qrow = (const bf16*)io.q + ((size_t)b * S + i_ld) * ldq + h * DK;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qf[kk] = *reinterpret_cast<const bf16x8*>(qrow + kk * 16 + g * 8);
    // (an empty use: the wait for these loads belongs here, not at their first use inside the loop, where it
    // would also wait for the tile DMA of every iteration -- see the dk/dv kernel)
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) asm volatile("" ::"v"(qf[kk]));
  }
  if constexpr (BIAS) {
    const float* dgh = diag + (size_t)h * (2 * S - 1);
    fill_bias_slice(dg, dgh, S + BR - 1, tid, [&](int t) {
      const int idx = t - (i0 + BR - 1) + (S - 1);  // delta + S - 1
      return idx < 0 ? 0 : idx;                     // only reachable by clamped (unused) queries
    });
  }
  const float sc = a.scale * kLog2e;
  const int dg_base = BR - 1 - i_loc;  // dg[dg_base + j] = bias(j - i)
  uint32_t k1 = 0;  // dropout row key of this lane's query
  if constexpr (DROP) k1 = drop_row_key(a.drop, (uint32_t)(((size_t)b * a.H + h) * S + i_ld));

  f32x16 oT[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct)
#pragma unroll
    for (int r = 0; r < 16; ++r) oT[ct][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  int n_kv = (Sk + BC - 1) / BC;
  if (CAUSAL) {
    const int last = (i0 + BR < S ? i0 + BR : S);
    n_kv = (last + BC - 1) / BC;
  }
  // K/V tiles are double buffered: tile jt+1 is in flight (DMA) while tile jt is used.  td_tail fetches the
  // last tile of a key sequence whose length is not a multiple of the tile.
  TileDma<DK, BC> td, td_tail;
  td.init(wave, lane, ld);
  td_tail.init(wave, lane, ld, Sk % BC ? Sk % BC : BC);
  const int jt_tail = Sk % BC ? Sk / BC : -1;  // index of the ragged tile, if there is one
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)smem;
  (jt_tail == 0 ? td_tail : td).issue(lds0, kbase, wave);
  (jt_tail == 0 ? td_tail : td).issue(lds0 + TILE, vbase, wave);
  for (int jt = 0; jt < n_kv; ++jt) {
    const int j0 = jt * BC;
    dma_wait_barrier();  // tile jt landed; every wave is done with the other stage
    if (jt + 1 < n_kv) {
      const uint32_t nxt = lds0 + ((jt + 1) & 1) * STG;
      const TileDma<DK, BC>& tn = jt + 1 == jt_tail ? td_tail : td;
      tn.issue(nxt, kbase + (size_t)(j0 + BC) * ld, wave);
      tn.issue(nxt + TILE, vbase + (size_t)(j0 + BC) * ld, wave);
    }
    const char* Kt = smem + (jt & 1) * STG;
    const char* Vt = Kt + TILE;

    f32x16 sT[BC / 32];
#pragma unroll
    for (int kt = 0; kt < BC / 32; ++kt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sT[kt][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KS; ++kk)
        sT[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<DK>(Kt, kt * 32, kk, lane), qf[kk], sT[kt],
                                                        0, 0, 0);
    }
    if constexpr (DK == 128) {
      // K operands requested two contraction steps ahead of the products that use them
      __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
#pragma unroll
      for (int q = 0; q + 3 < (BC / 32) * KS; ++q) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 3, 0);
    }
    float mx = -INFINITY;
    // only tiles that reach above the diagonal of this wave's queries pay for the mask (wave-uniform)
    // (and the tile that reaches past the last key)
    const bool on_diag = (CAUSAL && j0 + BC - 1 > i0 + wave * 32) || j0 + BC > Sk;
    if (on_diag) {
#pragma unroll
      for (int kt = 0; kt < BC / 32; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = j0 + kt * 32 + ((r >> 2) << 3) + (g << 2) + (r & 3);
          // (a masked key's bias slot may lie outside the slice: clamp the index, the value is discarded)
          const int jb = j < Sk ? j : Sk - 1;
          float s = BIAS ? fmaf(sT[kt][r], sc, dg[dg_base + jb]) : sT[kt][r] * sc;
          if ((CAUSAL && j > i) || j >= Sk) s = -INFINITY;
          sT[kt][r] = s;
          mx = fmaxf(mx, s);
        }
    } else {
#pragma unroll
      for (int kt = 0; kt < BC / 32; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = j0 + kt * 32 + ((r >> 2) << 3) + (g << 2) + (r & 3);
          const float s = BIAS ? fmaf(sT[kt][r], sc, dg[dg_base + j]) : sT[kt][r] * sc;
          sT[kt][r] = s;
          mx = fmaxf(mx, s);
        }
    }
    mx = max_across_halves(mx);
    const float m_new = fmaxf(m, mx);
    const float alpha = fast_exp2(m - m_new);
    m = m_new;
    float ls = 0.f;
#pragma unroll
    for (int kt = 0; kt < BC / 32; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = fast_exp2(sT[kt][r] - m_new);
        ls += p;  // the normaliser is that of the undropped probabilities
        if constexpr (DROP) {
          const int j = j0 + kt * 32 + ((r >> 2) << 3) + (g << 2) + (r & 3);
          sT[kt][r] = mix32(k1 ^ (uint32_t)j) >= a.drop.thr ? p : 0.f;
        } else {
          sT[kt][r] = p;
        }
      }
    l = l * alpha + ls;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int r = 0; r < 16; ++r) oT[ct][r] *= alpha;
#pragma unroll
    for (int kt = 0; kt < BC / 32; ++kt)
#pragma unroll
      for (int mm = 0; mm < 2; ++mm) {
        const bf16x8 pf = pack8(sT[kt], mm * 8);
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
          oT[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_tr<DK>(Vt, kt * 32 + mm * 16, ct * 32, lane),
                                                          pf, oT[ct], 0, 0, 0);
      }
  }
  const float l_tot = l + __shfl_xor(l, 32, 64);
  if (i < S) {
    const float inv = (DROP ? a.drop.scale : 1.f) / l_tot;
    bf16* crow = c + ((size_t)b * S + i) * I + h * DK;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (bf16)(oT[ct][rq * 4 + e] * inv);
        *reinterpret_cast<bf16x4*>(crow + ct * 32 + rq * 8 + g * 4) = o;
      }
    if (g == 0) lse[((size_t)b * a.H + h) * S + i] = (m + __builtin_amdgcn_logf(l_tot)) * kLn2;
  }
}

// ------------------------------------------------------------------------------------------------
// dq and the per-diagonal bias gradient.  Same ownership as the forward (lane = query).  The kernel also
// forms dvec[b,h,i] = sum_c dO[b,i,h,c] * O[b,i,h,c] for its query -- the two lane halves hold the two halves
// of the dO row as MFMA operands already, so it costs one read of the O row -- and writes it for the
// dk/dv kernel, which runs after this one.
//
// Bias gradient: ddiag[delta] = sum over (b, i) of ds[i, i + delta].  In the MFMA result layout a
// register holds one key offset for 32 queries, i.e. 32 consecutive diagonals, and a different
// register holds the same diagonals shifted by its key offset.  Rotating each register across the
// 32 lanes by its key offset (ds_swizzle rotate mode: a crossbar permute, no LDS memory) lines the
// diagonals up: after the rotation lane p holds, from every register, a value of diagonal slot
// 31 - p or 63 - p of the sub-tile's 63 diagonals.  Each lane therefore owns two slots per
// sub-tile, adds into them in a per-(wave, lane half) window in LDS with plain read-modify-write
// (the owner of a window entry never changes, so no synchronisation until the final flush), and the
// workgroup adds the eight windows up and issues one global atomic per diagonal.  Sub-tiles whose
// every offset lies in the saturated last bucket (|delta| >= far) skip all that and add into one
// scalar per lane; it is credited to the outermost diagonal, which is in the same bucket.
// ------------------------------------------------------------------------------------------------
template <int DK, bool CAUSAL, bool BIAS, bool DROP>
__global__ __launch_bounds__(256, DK == 64 && !DROP ? 3 : 2) void attn_bwd_dq_mfma_kernel(AttnIO io,
                                                               const bf16* __restrict__ o,
                                                               const bf16* __restrict__ dout,
                                                               const float* __restrict__ diag,
                                                               const float* __restrict__ lse,
                                                               float* __restrict__ dvec,
                                                               float* __restrict__ ddiag,
                                                               float* __restrict__ ddiag_part,
                                                               AttnDims a, int far) {
  constexpr int BR = 128, BC = 64, KS = DK / 16, CT = DK / 32;
  constexpr int TILE = BC * DK * 2, STG = 2 * TILE;  // a stage holds a K tile then a V tile
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  float* dg = reinterpret_cast<float*>(smem + 2 * STG);  // [S + BR - 1] bias, log2 units
  // Diagonal windows [4 waves][2 lane halves][W].  A sub-tile at key offset j0s - i_w0 = 32 m from
  // the wave's queries is resolved per diagonal for |m| <= nb; its slot u (0..62) lives at
  // (m + nb) * 32 + u, which is diagonal delta = 32 m + u - 31 (+ 4 for the upper lane half).
  const int nb = BIAS ? attn_dq_window_blocks(a.S, far) : 0, W = 32 * (2 * nb + 2);
  float* ddg_all = dg + (a.S + BR - 1);

  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int S = a.S, Sk = a.Sk, I = a.H * DK;
  const size_t ldq = (size_t)io.ldq, ld = (size_t)io.ldkv;
  int qt, h, b;
  decode_block((S + BR - 1) / BR, a.H, a.B, qt, h, b);
  if (CAUSAL) qt = (S + BR - 1) / BR - 1 - qt;
  const int i0 = qt * BR;
  const int i_w0 = i0 + wave * 32;         // first query of this wave
  const int i_lw = lane & 31;              // query index inside the wave
  const int i_loc = wave * 32 + i_lw;
  const int i = i0 + i_loc;
  const int i_ld = i < S ? i : S - 1;      // queries past the end read the last row; their ds is forced to zero
  const bool q_ok = i < S;
  const bf16* kbase = (const bf16*)io.k + (size_t)b * Sk * ld + h * DK;
  const bf16* vbase = (const bf16*)io.v + (size_t)b * Sk * ld + h * DK;
  float* ddgw = ddg_all + (wave * 2 + g) * W + (31 - i_lw);  // this lane's first slot of block m = -nb

  bf16x8 qf[KS], dof[KS];
  float dsum = 0.f;  // this lane half's share of sum_c dO * O
  {
    const bf16* qrow = (const bf16*)io.q + ((size_t)b * S + i_ld) * ldq + h * DK;
    const bf16* drow = dout + ((size_t)b * S + i_ld) * I + h * DK;
    const bf16* orow = o + ((size_t)b * S + i_ld) * I + h * DK;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      qf[kk] = *reinterpret_cast<const bf16x8*>(qrow + kk * 16 + g * 8);
      dof[kk] = *reinterpret_cast<const bf16x8*>(drow + kk * 16 + g * 8);
      const bf16x8 of = *reinterpret_cast<const bf16x8*>(orow + kk * 16 + g * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) dsum = fmaf((float)of[e], (float)dof[kk][e], dsum);
    }
    // (an empty use: see the forward kernel)
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) asm volatile("" ::"v"(qf[kk]), "v"(dof[kk]));
  }
  dsum += __shfl_xor(dsum, 32, 64);
  const size_t srow = ((size_t)b * a.H + h) * S + i_ld;
  // for the dk/dv kernel, which stages them per query tile by DMA: -dvec, and behind it -lse / scale
  const float lse_q = lse[srow];
  if (g == 0 && q_ok) {
    dvec[srow] = -dsum;
    dvec[(size_t)a.B * a.H * S + srow] = lse_q * (-1.f / a.scale);
  }
  const float nlse2 = -lse_q * kLog2e, ndv = -dsum;
  uint32_t k1 = 0;  // dropout row key of this lane's query
  if constexpr (DROP) k1 = drop_row_key(a.drop, (uint32_t)srow);
  // dP of a kept probability carries the factor 1/(1 - rate); that of a dropped one is zero
  auto dp_masked = [&](float dp, int j) {
    if constexpr (DROP) return mix32(k1 ^ (uint32_t)j) >= a.drop.thr ? dp * a.drop.scale : 0.f;
    else return dp;
  };
  if constexpr (BIAS) {
    const float* dgh = diag + (size_t)h * (2 * S - 1);
    fill_bias_slice(dg, dgh, S + BR - 1, tid, [&](int t) {
      const int idx = t - (i0 + BR - 1) + (S - 1);  // delta + S - 1
      return idx < 0 ? 0 : idx;                     // only reachable by queries past the end
    });
    for (int t = tid; t < 8 * W; t += 256) ddg_all[t] = 0.f;
  }
  const float sc = a.scale * kLog2e;
  const int dg_base = BR - 1 - i_loc;
  float far_neg = 0.f, far_pos = 0.f;

  f32x16 dqT[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct)
#pragma unroll
    for (int r = 0; r < 16; ++r) dqT[ct][r] = 0.f;

  const int n_kv = ((CAUSAL && i0 + BR < Sk ? i0 + BR : Sk) + BC - 1) / BC;
  TileDma<DK, BC> td, td_tail;  // td_tail: the last tile of a key sequence that does not fill it
  td.init(wave, lane, ld);
  td_tail.init(wave, lane, ld, Sk % BC ? Sk % BC : BC);
  const int jt_tail = Sk % BC ? Sk / BC : -1;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)smem;
  (jt_tail == 0 ? td_tail : td).issue(lds0, kbase, wave);
  (jt_tail == 0 ? td_tail : td).issue(lds0 + TILE, vbase, wave);
  for (int jt = 0; jt < n_kv; ++jt) {
    const int j0 = jt * BC;
    dma_wait_barrier();  // tile jt landed; every wave is done with the other stage
    if (jt + 1 < n_kv) {
      const uint32_t nxt = lds0 + ((jt + 1) & 1) * STG;
      const TileDma<DK, BC>& tn = jt + 1 == jt_tail ? td_tail : td;
      tn.issue(nxt, kbase + (size_t)(j0 + BC) * ld, wave);
      tn.issue(nxt + TILE, vbase + (size_t)(j0 + BC) * ld, wave);
    }
    const char* Kt = smem + (jt & 1) * STG;
    const char* Vt = Kt + TILE;
#pragma unroll
    for (int kt = 0; kt < BC / 32; ++kt) {
      const int j0s = j0 + kt * 32;
      if (CAUSAL && j0s > i_w0 + 31) continue;  // whole sub-tile masked for this wave
      if (j0s >= Sk || i_w0 >= S) continue;     // whole sub-tile past the last key, or no query of this wave exists
      // The bias values are requested before the MFMAs (and the scheduler may not sink them): read at
      // first use, each one stalls the softmax arithmetic for an LDS round trip.  Prefetching the
      // MFMA operands as well, or seeding the accumulators with -lse and -dvec, costs more registers
      // than the third wave per SIMD they displace is worth (measured).
      float bias[16];
      if constexpr (BIAS) {
        if (j0s + 32 <= Sk) {
          // every key of the sub-tile exists: one address per lane and sixteen constant offsets (with the
          // clamp below each value costs four address instructions, a third of the kernel's vector work)
          const float* bp = dg + (dg_base + j0s + (g << 2));
#pragma unroll
          for (int r = 0; r < 16; ++r) bias[r] = bp[((r >> 2) << 3) + (r & 3)];
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = j0s + ((r >> 2) << 3) + (g << 2) + (r & 3);
            bias[r] = dg[dg_base + (j < Sk ? j : Sk - 1)];  // (keys past the end are masked below)
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      f32x16 sT, dpT;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sT[r] = 0.f; dpT[r] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        sT = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<DK>(Kt, kt * 32, kk, lane), qf[kk], sT, 0, 0, 0);
        dpT = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows<DK>(Vt, kt * 32, kk, lane), dof[kk], dpT, 0, 0, 0);
      }
      // the K / V operands of a contraction step are requested one step ahead of the products that use them
      // (left alone the compiler reads them right before, and every pair of products waits out an LDS round trip)
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int kk = 0; kk + 2 < KS; ++kk) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      // sub-tile reaches above the diagonal, past the last key, or this wave holds queries past the end
      // (all wave-uniform)
      if ((CAUSAL && j0s + 31 > i_w0) || j0s + 32 > Sk || i_w0 + 32 > S) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = j0s + ((r >> 2) << 3) + (g << 2) + (r & 3);
          float p = BIAS ? fast_exp2(fmaf(sT[r], sc, bias[r]) + nlse2) : fast_exp2(fmaf(sT[r], sc, nlse2));
          if ((CAUSAL && j > i) || j >= Sk || !q_ok) p = 0.f;
          sT[r] = p * (dp_masked(dpT[r], j) + ndv);
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = j0s + ((r >> 2) << 3) + (g << 2) + (r & 3);
          const float p = BIAS ? fast_exp2(fmaf(sT[r], sc, bias[r]) + nlse2) : fast_exp2(fmaf(sT[r], sc, nlse2));
          sT[r] = p * (dp_masked(dpT[r], j) + ndv);
        }
      }
      // ---- bias gradient of this 32x32 sub-tile (wave-uniform branches)
      if constexpr (!BIAS) {
      } else if (j0s + 31 - i_w0 <= -far) {
        float t = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) t += sT[r];
        far_neg += t;
      } else if (!CAUSAL && j0s - i_w0 - 31 >= far) {
        float t = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) t += sT[r];
        far_pos += t;
      } else {
        float lo = 0.f, tot = 0.f;
        diag_accum(sT, 31 - i_lw, lo, tot);
        float* slot = ddgw + ((j0s - i_w0) / 32 + nb) * 32;
        slot[0] += lo;
        slot[32] += tot - lo;
      }
#pragma unroll
      for (int mm = 0; mm < 2; ++mm) {
        const bf16x8 dsf = pack8(sT, mm * 8);
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
          dqT[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              frag_cols_tr<DK>(Kt, kt * 32 + mm * 16, ct * 32, lane), dsf, dqT[ct], 0, 0, 0);
      }
    }
  }
  if (q_ok) {
    bf16* qrow = (bf16*)io.dq + ((size_t)b * S + i) * (size_t)io.lddq + h * DK;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (bf16)(dqT[ct][rq * 4 + e] * a.scale);
        *reinterpret_cast<bf16x4*>(qrow + ct * 32 + rq * 8 + g * 4) = o;
      }
  }
  if constexpr (!BIAS) return;
  // ---- flush: add the eight windows up (the upper lane half's diagonals sit 4 higher) and either issue one
  // global atomic per diagonal of this workgroup or, for a reproducible result, write the summed window to
  // this workgroup's row of ddiag_part (attn_ddiag_reduce_kernel adds the rows up in a fixed order)
  float* ddh = ddiag + (size_t)h * (2 * S - 1);
  float* part = nullptr;
  if (ddiag_part) part = ddiag_part + (((size_t)b * a.H + h) * ((S + BR - 1) / BR) + qt) * (size_t)attn_ddiag_part_stride(S);
  __syncthreads();
  for (int t = tid; t < W + 4; t += 256) {
    float v = 0.f;
#pragma unroll
    for (int wv = 0; wv < 4; ++wv) {
      if (t < W) v += ddg_all[(wv * 2) * W + t];
      if (t >= 4) v += ddg_all[(wv * 2 + 1) * W + t - 4];
    }
    // window entry t of wave wv: delta = t - 32 nb - 31 relative to that wave's first query, and
    // the waves' first queries are 32 apart -- but so are their windows' origins (m counts from the
    // wave's own queries), so the entry means the same diagonal for every wave
    const int idx = t - 32 * nb - 31 + (S - 1);
    if (part) part[t] = v;
    else if (v != 0.f && idx >= 0 && idx < 2 * S - 1) unsafeAtomicAdd(&ddh[idx], v);
  }
  far_neg = wave_sum(far_neg);
  far_pos = wave_sum(far_pos);
  if (part) {
    // per-wave sums, added by one lane in wave order
    float* fs = ddg_all;  // the windows have been read
    __syncthreads();
    if (lane == 0) { fs[wave * 2] = far_neg; fs[wave * 2 + 1] = far_pos; }
    __syncthreads();
    if (tid == 0) {
      part[W + 4] = (fs[0] + fs[2]) + (fs[4] + fs[6]);
      part[W + 5] = (fs[1] + fs[3]) + (fs[5] + fs[7]);
    }
  } else if (lane == 0) {
    if (far_neg != 0.f) unsafeAtomicAdd(&ddh[0], far_neg);
    if (far_pos != 0.f) unsafeAtomicAdd(&ddh[2 * S - 2], far_pos);
  }
}

// ddiag[h][..] += the window rows that the dq workgroups of head h wrote, always in the same order: a thread
// owns one window entry (or one of the two saturated-bucket sums behind the window), four threads share the
// rows (row r goes to thread group r % 4) and their sums are added in group order.  Where the window reaches an
// end diagonal, the saturated-bucket sum of that end lands on the same address: the window entry's thread adds
// both, so no two threads ever update one address.
__global__ __launch_bounds__(256) void attn_ddiag_reduce_kernel(const float* __restrict__ part,
                                                              float* __restrict__ ddiag, int B, int H, int S,
                                                              int nb) {
  __shared__ float red[2][4][64];
  const int nch = gridDim.x / H;
  const int h = blockIdx.x / nch, chunk = blockIdx.x % nch;
  const int nt = (S + 127) / 128, W = 32 * (2 * nb + 2), rows = B * nt;
  const size_t stride = (size_t)attn_ddiag_part_stride(S);
  const int tl = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int t = chunk * 64 + tl;                      // entry: [0, W+4) window, W+4 / W+5 the two sums
  const int last = 2 * S - 2;
  int idx = -1;
  if (t < W + 4) idx = t - 32 * nb - 31 + (S - 1);
  else if (t == W + 4) idx = 0;
  else if (t == W + 5) idx = last;
  const bool valid = idx >= 0 && idx <= last;
  // does a window entry own this end?  (entry t0 maps to diagonal 0, entry t1 to the last one)
  const int t0 = 32 * nb + 31 - (S - 1), t1 = t0 + last;
  const bool win0 = t0 >= 0 && t0 < W + 4, win1 = t1 >= 0 && t1 < W + 4;
  int extra = -1;                                      // second column this thread adds
  if (t < W + 4 && idx == 0) extra = W + 4;
  if (t < W + 4 && idx == last) extra = W + 5;
  const bool skip = (t == W + 4 && win0) || (t == W + 5 && win1);
  float s = 0.f, s2 = 0.f;
  if (valid && !skip) {
    // rows of head h: (b, q) -> ((b*H + h)*nt + q)
    for (int r = grp; r < rows; r += 4) {
      const size_t base = (((size_t)(r / nt) * H + h) * nt + r % nt) * stride;
      s += part[base + t];
      if (extra >= 0) s2 += part[base + extra];
    }
  }
  red[0][grp][tl] = s;
  red[1][grp][tl] = s2;
  __syncthreads();
  if (grp == 0 && valid && !skip) {
    const float tot = ((red[0][0][tl] + red[0][1][tl]) + (red[0][2][tl] + red[0][3][tl])) +
                      ((red[1][0][tl] + red[1][1][tl]) + (red[1][2][tl] + red[1][3][tl]));
    ddiag[(size_t)h * (2 * S - 1) + idx] += tot;
  }
}

// ------------------------------------------------------------------------------------------------
// dk and dv.  grid (Sk/128) * H * B; wave w owns keys j0 + 32w + lane%32; loops over query tiles.
// ------------------------------------------------------------------------------------------------
template <int DK, bool CAUSAL, bool BIAS, bool DROP>
__global__ __launch_bounds__(256, DK == 64 ? 2 : 1) void attn_bwd_dkv_mfma_kernel(AttnIO io,
                                                                const bf16* __restrict__ dout,
                                                                const float* __restrict__ diag,
                                                                const float* __restrict__ lse,
                                                                const float* __restrict__ dvec,
                                                                AttnDims a) {
  constexpr int BCK = 128, BQ = 64, KS = DK / 16, CT = DK / 32;
  constexpr int TILE = BQ * DK * 2, STG = 2 * TILE;  // a stage holds a Q tile then a dO tile
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  // The score and dP accumulators start from -lse/scale and -dvec, so that the MFMA results are
  // already (s - lse/scale) and (dP - dvec): no per-element subtraction afterwards.
  float* lse_all = reinterpret_cast<float*>(smem + 2 * STG);  // [2 stages][BQ]  -lse / scale
  float* dv_all = lse_all + 2 * BQ;                           // [2 stages][BQ]  -dvec
  uint32_t* key_all = reinterpret_cast<uint32_t*>(dv_all + 2 * BQ);  // [2 stages][BQ] dropout row keys (DROP only)
  // [-BQ, S + BCK - 1) log2 units (BIAS only); the BQ entries in front are only ever read for queries past the
  // end of a ragged last tile, whose probabilities are set to zero
  float* dg = dv_all + 2 * BQ + (DROP ? 2 * BQ : 0) + BQ;

  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int S = a.S, Sk = a.Sk, I = a.H * DK;
  const size_t ld = (size_t)io.ldq, ldkv = (size_t)io.ldkv;
  int kt_, h, b;
  decode_block((Sk + BCK - 1) / BCK, a.H, a.B, kt_, h, b);
  const int j0 = kt_ * BCK;
  const int j_loc = wave * 32 + (lane & 31);
  const int j = j0 + j_loc;
  const int j_ld = j < Sk ? j : Sk - 1;
  const bf16* base = (const bf16*)io.q + (size_t)b * S * ld + h * DK;
  const bf16* dobase = dout + (size_t)b * S * I + h * DK;

  bf16x8 kf[KS], vf[KS];
  {
    const bf16* krow = (const bf16*)io.k + ((size_t)b * Sk + j_ld) * ldkv + h * DK;
    const bf16* vrow = (const bf16*)io.v + ((size_t)b * Sk + j_ld) * ldkv + h * DK;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      kf[kk] = *reinterpret_cast<const bf16x8*>(krow + kk * 16 + g * 8);
      vf[kk] = *reinterpret_cast<const bf16x8*>(vrow + kk * 16 + g * 8);
    }
    // The compiler waits for these loads where they are first used, and that is inside the loop: its
    // s_waitcnt vmcnt(n) there would run in every iteration and, since the counter also counts the tile DMA
    // issued at the top of the iteration, stall the first matrix instructions until the whole DMA has landed.
    // An empty use here moves the wait in front of the loop.
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) asm volatile("" ::"v"(kf[kk]), "v"(vf[kk]));
  }
  if constexpr (BIAS) {
    // dg[t] = bias(delta) for delta = t + j0 - (S - 1), t in [0, S + BCK - 1)
    const float* dgh = diag + (size_t)h * (2 * S - 1);
    for (int t = tid; t < S + BCK - 1; t += 256) {
      int idx = t + j0;  // delta + S - 1
      idx = idx > 2 * S - 2 ? 2 * S - 2 : idx;
      dg[t] = dgh[idx] * kLog2e;
    }
    if (tid < BQ) dg[tid - BQ] = 0.f;
  }
  const float sc = a.scale * kLog2e;
  // dg index of (query i, key j): (j - i) - (j0 - (S-1)) = j_loc + (S - 1 - i)
  f32x16 dkT[CT], dvT[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dkT[ct][r] = 0.f; dvT[ct][r] = 0.f; }

  const int it_begin = CAUSAL ? (j0 / BQ) : 0;
  const size_t srow = ((size_t)b * a.H + h) * S;
  // Q/dO tiles (DMA) and the matching lse / dvec slices are double buffered.
  // tq_tail / tdo_tail: the last tile of a query sequence that does not fill it
  TileDma<DK, BQ> tq, tdo, tq_tail, tdo_tail;
  tq.init(wave, lane, ld);
  tdo.init(wave, lane, (size_t)I);
  tq_tail.init(wave, lane, ld, S % BQ ? S % BQ : BQ);
  tdo_tail.init(wave, lane, (size_t)I, S % BQ ? S % BQ : BQ);
  const int it_tail = S % BQ ? S / BQ : -1;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)smem;
  const int n_it = (S + BQ - 1) / BQ;
  (it_begin == it_tail ? tq_tail : tq).issue(lds0, base + (size_t)it_begin * BQ * ld, wave);
  (it_begin == it_tail ? tdo_tail : tdo).issue(lds0 + TILE, dobase + (size_t)it_begin * BQ * I, wave);
  // The -lse / scale and -dvec slices of a query tile (written by the dq kernel) travel by DMA as well, one
  // instruction each from waves 0 and 1.  Fetched with ordinary loads they put compiler-made vmcnt waits into
  // the loop, and since those count the tile DMA issued just before them, every iteration waited out the
  // whole DMA latency at its first matrix instruction.
  const float* ndvec = dvec + srow;
  const float* nlse = dvec + (size_t)a.B * a.H * S + srow;
  const uint32_t lds_lse = lds0 + 2 * STG, lds_dv = lds_lse + 2 * BQ * 4;
  auto issue_rows = [&](int stage, int q_first) __attribute__((always_inline)) {
    const int qi = q_first + lane < S ? q_first + lane : S - 1;  // (rows past the end are masked)
    if (wave == 0) dma_64f(lds_lse + stage * BQ * 4, nlse, (uint32_t)qi * 4u);
    if (wave == 1) dma_64f(lds_dv + stage * BQ * 4, ndvec, (uint32_t)qi * 4u);
  };
  issue_rows(0, it_begin * BQ);
  if constexpr (DROP) {
    if (tid < BQ) {
      const int qi = it_begin * BQ + tid < S ? it_begin * BQ + tid : S - 1;
      key_all[tid] = drop_row_key(a.drop, (uint32_t)(srow + qi));
    }
  }
  for (int it = it_begin; it < n_it; ++it) {
    const int q0 = it * BQ;
    const int st = (it - it_begin) & 1;
    dma_wait_barrier();  // tile `it` and its lse / dvec slices landed; other stage is free
    uint32_t nkey = 0;
    const bool more = it + 1 < n_it;
    if (more) {
      const uint32_t nxt = lds0 + (st ^ 1) * STG;
      (it + 1 == it_tail ? tq_tail : tq).issue(nxt, base + (size_t)(q0 + BQ) * ld, wave);
      (it + 1 == it_tail ? tdo_tail : tdo).issue(nxt + TILE, dobase + (size_t)(q0 + BQ) * I, wave);
      issue_rows(st ^ 1, q0 + BQ);
      if constexpr (DROP) {
        if (tid < BQ) {
          const int qi = q0 + BQ + tid < S ? q0 + BQ + tid : S - 1;
          nkey = drop_row_key(a.drop, (uint32_t)(srow + qi));
        }
      }
    }
    const char* Qt = smem + st * STG;
    const char* Dt = Qt + TILE;
    const float* lse_s = lse_all + st * BQ;
    const float* dv_s = dv_all + st * BQ;
    const uint32_t* key_s = key_all + st * BQ;
    bf16x8 qr[KS], dr[KS];
#pragma unroll
    for (int qb = 0; qb < BQ / 32; ++qb) {
      // bias values and accumulator seeds are requested before the MFMAs so that their LDS latency
      // is hidden behind the matrix work instead of stalling the softmax arithmetic (read at first use they
      // put an LDS round trip on every sub-tile's dependent chain: 651 -> 635 us at 64 channels, the sixteen
      // registers are there at two waves per SIMD)
      constexpr bool HOIST = BIAS;
      float bias[16];
      // Bias of (query i, key j) sits at dg[j_loc + S - 1 - i].  Where every query of the tile exists the sixteen
      // values of a lane are one pointer and constant offsets: register r belongs to query
      // q0 + qb*32 + 4g + c_r with c_r = 8*(r/4) + r%4 <= 27, so bq[27 - c_r] with bq 27 below the first.
      // (a query past the end of a ragged tile reads at most BQ - 1 entries below dg[0]: the padding)
      const float* bq = dg + (j_loc + S - 1 - q0 - qb * 32 - (g << 2) - 27);
      if constexpr (HOIST) {
#pragma unroll
        for (int r = 0; r < 16; ++r) bias[r] = bq[27 - (((r >> 2) << 3) + (r & 3))];
      }
      f32x16 s, dp;
      // likewise the row operands of the tile's second sub-tile, requested before the dV / dK products of
      // the first
      constexpr bool ROWS_AHEAD = DK == 128;
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_s + qb * 32 + rq * 8 + g * 4);
        const f32x4 d4 = *reinterpret_cast<const f32x4*>(dv_s + qb * 32 + rq * 8 + g * 4);
#pragma unroll
        // with dropout dP is rescaled before dvec is subtracted: it starts from zero
        for (int e = 0; e < 4; ++e) { s[rq * 4 + e] = l4[e]; dp[rq * 4 + e] = DROP ? 0.f : d4[e]; }
      }
      if constexpr (HOIST) __builtin_amdgcn_sched_group_barrier(0x100, 12, 0);  // 8 bias + 4 seed reads first
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        const bool pre = ROWS_AHEAD && qb == 1;
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pre ? qr[kk] : frag_rows<DK>(Qt, qb * 32, kk, lane), kf[kk], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pre ? dr[kk] : frag_rows<DK>(Dt, qb * 32, kk, lane), vf[kk], dp, 0, 0, 0);
      }

      // with 128 channels (one wave per SIMD, registers to spare) the transposed Q and dO operands of the
      // dV / dK products are requested before the softmax arithmetic, which then covers their LDS
      // latency; with 64 channels the second wave on the SIMD covers it and the registers are not there
      constexpr bool TR_AHEAD = DK == 128;
      bf16x8 dtr[2][CT], qtr[2][CT];
      if constexpr (TR_AHEAD) {
#pragma unroll
        for (int mm = 0; mm < 2; ++mm)
#pragma unroll
          for (int ct = 0; ct < CT; ++ct) {
            dtr[mm][ct] = frag_cols_tr<DK>(Dt, qb * 32 + mm * 16, ct * 32, lane);
            qtr[mm][ct] = frag_cols_tr<DK>(Qt, qb * 32 + mm * 16, ct * 32, lane);
          }
      }
      // with 64 channels the second copy of the loop costs a wave per SIMD in registers: mask always
      // some key here lies after some query, or the tile reaches past the last query (both wave-uniform)
      if ((CAUSAL && (DK == 64 || j0 + wave * 32 + 31 > q0 + qb * 32)) || q0 + BQ > S) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int il = qb * 32 + ((r >> 2) << 3) + (g << 2) + (r & 3);
          const int i = q0 + il;
          float p = BIAS ? fast_exp2(fmaf(s[r], sc, HOIST ? bias[r] : bq[27 - (((r >> 2) << 3) + (r & 3))]))
                         : fast_exp2(s[r] * sc);
          if ((CAUSAL && j > i) || i >= S) p = 0.f;
          if constexpr (DROP) {
            const bool keep = mix32(key_s[il] ^ (uint32_t)j) >= a.drop.thr;
            s[r] = keep ? p : 0.f;
            dp[r] = p * ((keep ? dp[r] * a.drop.scale : 0.f) + dv_s[il]);
          } else {
            s[r] = p;
            dp[r] = p * dp[r];
          }
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int il = qb * 32 + ((r >> 2) << 3) + (g << 2) + (r & 3);
          const int i = q0 + il;
          const float p = BIAS ? fast_exp2(fmaf(s[r], sc, HOIST ? bias[r] : bq[27 - (((r >> 2) << 3) + (r & 3))]))
                               : fast_exp2(s[r] * sc);
          if constexpr (DROP) {
            const bool keep = mix32(key_s[il] ^ (uint32_t)j) >= a.drop.thr;
            s[r] = keep ? p : 0.f;
            dp[r] = p * ((keep ? dp[r] * a.drop.scale : 0.f) + dv_s[il]);
          } else {
            s[r] = p;
            dp[r] = p * dp[r];
          }
        }
      }
      if constexpr (ROWS_AHEAD) {
        if (qb == 0) {
#pragma unroll
          for (int kk = 0; kk < KS; ++kk) {
            qr[kk] = frag_rows<DK>(Qt, 32, kk, lane);
            dr[kk] = frag_rows<DK>(Dt, 32, kk, lane);
          }
        }
      }
#pragma unroll
      for (int mm = 0; mm < 2; ++mm) {
        const bf16x8 pf = pack8(s, mm * 8), dsf = pack8(dp, mm * 8);
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
          dvT[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              TR_AHEAD ? dtr[mm][ct] : frag_cols_tr<DK>(Dt, qb * 32 + mm * 16, ct * 32, lane), pf, dvT[ct], 0, 0, 0);
          dkT[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              TR_AHEAD ? qtr[mm][ct] : frag_cols_tr<DK>(Qt, qb * 32 + mm * 16, ct * 32, lane), dsf, dkT[ct], 0, 0, 0);
        }
      }
    }
    if constexpr (DROP) {
      if (more && tid < BQ) key_all[(st ^ 1) * BQ + tid] = nkey;
    }
  }
  if (j < Sk) {
    bf16* krow = (bf16*)io.dk + ((size_t)b * Sk + j) * (size_t)io.lddkv + h * DK;
    bf16* vrow = (bf16*)io.dv + ((size_t)b * Sk + j) * (size_t)io.lddkv + h * DK;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        bf16x4 ok, ov;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          ok[e] = (bf16)(dkT[ct][rq * 4 + e] * a.scale);
          ov[e] = (bf16)(DROP ? dvT[ct][rq * 4 + e] * a.drop.scale : dvT[ct][rq * 4 + e]);
        }
        *reinterpret_cast<bf16x4*>(krow + ct * 32 + rq * 8 + g * 4) = ok;
        *reinterpret_cast<bf16x4*>(vrow + ct * 32 + rq * 8 + g * 4) = ov;
      }
  }
}

size_t attn_bwd_dq_lds_bytes(const AttnDims& a, int far) {
  if (!a.bias) return (size_t)4 * 64 * a.dk * 2;
  const int W = 32 * (2 * attn_dq_window_blocks(a.S, far) + 2);
  return (size_t)4 * 64 * a.dk * 2 + sizeof(float) * ((size_t)(a.S + 127) + 8 * (size_t)W);
}

template <typename K>
hipError_t set_lds(K kern, size_t bytes) {
  return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

template <int DK, bool CAUSAL, bool BIAS, bool DROP = false>
hipError_t fwd_launch(const AttnIO& io, const float* diag, void* c, float* lse, const AttnDims& a, hipStream_t st) {
  auto kern = attn_fwd_mfma_kernel<DK, CAUSAL, BIAS, DROP>;
  const size_t lds = 4 * 64 * DK * 2 + (BIAS ? sizeof(float) * (a.S + 127) : 0);
  hipError_t e = set_lds(kern, lds);
  if (e != hipSuccess) return e;
  kern<<<dim3(((a.S + 127) / 128) * a.H * a.B), 256, lds, st>>>(io, diag, (bf16*)c, lse, a);
  return hipGetLastError();
}

template <int DK, bool CAUSAL, bool BIAS, bool DROP = false>
hipError_t bwd_launch(const AttnIO& io, const void* c, const void* dc, const float* diag, const float* lse,
                      float* dvec, float* ddiag, float* ddiag_part, const AttnDims& a, int far, int phase,
                      hipStream_t st) {
  hipError_t e = hipSuccess;
  if (phase == 1) {
    auto kern = attn_bwd_dq_mfma_kernel<DK, CAUSAL, BIAS, DROP>;
    const size_t lds = attn_bwd_dq_lds_bytes(a, far);
    if ((e = set_lds(kern, lds)) != hipSuccess) return e;
    kern<<<dim3(((a.S + 127) / 128) * a.H * a.B), 256, lds, st>>>(io, (const bf16*)c, (const bf16*)dc, diag, lse, dvec, ddiag,
                                                          BIAS ? ddiag_part : nullptr, a, far);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (BIAS && ddiag_part) {
      const int nb = attn_dq_window_blocks(a.S, far);
      attn_ddiag_reduce_kernel<<<a.H * ceil_div(32 * (2 * nb + 2) + 6, 64), 256, 0, st>>>(ddiag_part, ddiag, a.B, a.H,
                                                                                         a.S, nb);
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
  }
  if (phase == 2) {
    auto kern = attn_bwd_dkv_mfma_kernel<DK, CAUSAL, BIAS, DROP>;
    const size_t lds = 4 * 64 * DK * 2 + sizeof(float) * (256 + (DROP ? 128 : 0) + (BIAS ? 64 + a.S + 127 : 0));
    if ((e = set_lds(kern, lds)) != hipSuccess) return e;
    kern<<<dim3(((a.Sk + 127) / 128) * a.H * a.B), 256, lds, st>>>(io, (const bf16*)dc, diag, lse, dvec, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  return hipSuccess;
}

// 0: self-attention with bias, 1: the same with the causal mask, 2: cross-attention (no bias, no mask)
int attn_mode(const AttnDims& a) { return a.bias ? (a.causal ? 1 : 0) : 2; }

}  // namespace

bool attn_bwd_mfma_fits(const AttnDims& a, int far) {
  // the dq kernel keeps per-diagonal windows of about 2 * far entries in LDS
  return attn_bwd_dq_lds_bytes(a, far < 1 ? 1 : far) <= (size_t)150 * 1024;
}

bool attn_mfma_supported(const AttnDims& a) {
  // Any lengths from 32 up (tiles are rounded up and their tails masked); LDS holds the diagonal slice
  // (S + 127 floats).  Without the bias only the unmasked form exists; bias and mask need square scores.
  if (!(a.dk == 64 || a.dk == 128) || a.S < 32 || a.Sk < 32 || a.S > 8192 || a.Sk > 65536) return false;
  if (a.bias) return a.Sk == a.S;
  return !a.causal;
}

hipError_t launch_attn_fwd_mfma(const AttnIO& io, const float* diag, void* c, float* lse, const AttnDims& a,
                                hipStream_t st) {
  if (!attn_mfma_supported(a)) return hipErrorInvalidValue;
  const int mode = attn_mode(a);
  if (a.drop.on) {
    if (a.dk == 64) {
      if (mode == 0) return fwd_launch<64, false, true, true>(io, diag, c, lse, a, st);
      if (mode == 1) return fwd_launch<64, true, true, true>(io, diag, c, lse, a, st);
      return fwd_launch<64, false, false, true>(io, diag, c, lse, a, st);
    }
    if (mode == 0) return fwd_launch<128, false, true, true>(io, diag, c, lse, a, st);
    if (mode == 1) return fwd_launch<128, true, true, true>(io, diag, c, lse, a, st);
    return fwd_launch<128, false, false, true>(io, diag, c, lse, a, st);
  }
  if (a.dk == 64) {
    if (mode == 0) return fwd_launch<64, false, true>(io, diag, c, lse, a, st);
    if (mode == 1) return fwd_launch<64, true, true>(io, diag, c, lse, a, st);
    return fwd_launch<64, false, false>(io, diag, c, lse, a, st);
  }
  if (mode == 0) return fwd_launch<128, false, true>(io, diag, c, lse, a, st);
  if (mode == 1) return fwd_launch<128, true, true>(io, diag, c, lse, a, st);
  return fwd_launch<128, false, false>(io, diag, c, lse, a, st);
}

size_t attn_ddiag_part_bytes(const AttnDims& a) {
  return (size_t)a.B * a.H * ((a.S + 127) / 128) * (size_t)attn_ddiag_part_stride(a.S) * sizeof(float);
}

hipError_t launch_attn_bwd_mfma(const AttnIO& io, const void* c, const void* dc, const float* diag,
                                const float* lse, float* dvec, float* ddiag, const AttnDims& a, int far,
                                int phase, hipStream_t st, float* ddiag_part) {
  // phase 1: dq, dvec = rowsum(dO * O) and the bias-gradient diagonals (added into ddiag); phase 2: dk, dv
  // (reads the dvec phase 1 wrote).
  // `far`: smallest distance that falls in the last (saturated) bucket; such offsets need no
  // per-diagonal resolution.  Never below 1, so offset 0 always takes the per-diagonal path.
  if (!attn_mfma_supported(a)) return hipErrorInvalidValue;
  if (far < 1) far = 1;
  const int mode = attn_mode(a);
  if (a.drop.on) {
    if (a.dk == 64) {
      if (mode == 0) return bwd_launch<64, false, true, true>(io, c, dc, diag, lse, dvec, ddiag, ddiag_part, a, far, phase, st);
      if (mode == 1) return bwd_launch<64, true, true, true>(io, c, dc, diag, lse, dvec, ddiag, ddiag_part, a, far, phase, st);
      return bwd_launch<64, false, false, true>(io, c, dc, diag, lse, dvec, ddiag, ddiag_part, a, far, phase, st);
    }
    if (mode == 0) return bwd_launch<128, false, true, true>(io, c, dc, diag, lse, dvec, ddiag, ddiag_part, a, far, phase, st);
    if (mode == 1) return bwd_launch<128, true, true, true>(io, c, dc, diag, lse, dvec, ddiag, ddiag_part, a, far, phase, st);
    return bwd_launch<128, false, false, true>(io, c, dc, diag, lse, dvec, ddiag, ddiag_part, a, far, phase, st);
  }
  if (a.dk == 64) {
    if (mode == 0) return bwd_launch<64, false, true>(io, c, dc, diag, lse, dvec, ddiag, ddiag_part, a, far, phase, st);
    if (mode == 1) return bwd_launch<64, true, true>(io, c, dc, diag, lse, dvec, ddiag, ddiag_part, a, far, phase, st);
    return bwd_launch<64, false, false>(io, c, dc, diag, lse, dvec, ddiag, ddiag_part, a, far, phase, st);
  }
  if (mode == 0) return bwd_launch<128, false, true>(io, c, dc, diag, lse, dvec, ddiag, ddiag_part, a, far, phase, st);
  if (mode == 1) return bwd_launch<128, true, true>(io, c, dc, diag, lse, dvec, ddiag, ddiag_part, a, far, phase, st);
  return bwd_launch<128, false, false>(io, c, dc, diag, lse, dvec, ddiag, ddiag_part, a, far, phase, st);
}

}  // namespace t5mi
