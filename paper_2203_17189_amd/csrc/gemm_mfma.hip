// bf16 MFMA GEMM for gfx950 (v_mfma_f32_32x32x16_bf16, float32 accumulation) with fused epilogues.
//
//   C[m,n] = sum_s sum_k A_s(m,k) B_s(n,k)
//
// Tiling: workgroup tile BM x BN, k-tiles of BK, WM x WN wavefronts, each wave owns
// (BM/WM) x (BN/WN) as 32x32 MFMA tiles.  BK = 64 in two stages for the large k-contiguous problems (a
// DMA request then covers a whole 128-byte line of a row; with 64-byte rows the L1 still spends a
// line's worth of time per request), BK = 32 in three to five stages elsewhere.
//
// Data path: global -> LDS directly (global_load_lds_dwordx4: every lane fetches 16 bytes, a wave
// fills 1 KB of contiguous LDS), NS stages deep.  Global load latency on this part is on the order
// of a microsecond under load while one k-tile is ~0.4 us of MFMA work, so several k-tiles must be
// in flight; keeping them in LDS instead of registers leaves the register file to the accumulators.
// Because the DMA writes LDS linearly, the bank-conflict swizzle is applied on the global side: the
// lane that owns LDS slot (row, physical chunk) fetches the logical chunk that belongs there.
// Two operand layouts:
//   k-contiguous (A[m][k]):  LDS rows of BK k (64 or 128 B: 4 or 8 chunks), read with ds_read_b128;
//   m-contiguous (A[k][m]):  LDS rows of BM m, 32-byte granules swizzled by k, read with the LDS
//                            transpose load ds_read_b64_tr_b16 (two per MFMA operand).
// The compiler does not see these DMA writes; ordering is explicit: s_waitcnt vmcnt(n) + s_barrier
// before a stage is read, and a stage is refilled only after a barrier that every wave reaches
// after its last read of that stage.
// Workgroup ids are remapped so that each XCD (ids are dealt round-robin to the 8 XCDs) works on a
// compact block of output tiles and shares operand tiles through its own L2.
#include "kernels.h"
#include <atomic>
#include <type_traits>

namespace t5mi {

namespace {

constexpr int KQ = 64;   // every segment's K must be a multiple of this

typedef __attribute__((address_space(3))) short4v lds_short4;

// k-contiguous stage: row r (BK*2 bytes) holds logical 16-byte chunk c at physical chunk c ^ kc_swz(r).
template <int BK>
__device__ __forceinline__ int kc_swz(int row) {
  if constexpr (BK == 32) return ((row >> 1) & 3) ^ ((row >> 3) & 1);
  else return (row ^ (row >> 3)) & 7;
}

// One MFMA operand (8 bf16 of k for row base + lane%32) for k-step kk of a stage.
template <int ROWS, bool KC, int BK>
__device__ __forceinline__ bf16x8 load_frag(const char* stage, int base, int kk, int lane) {
  if constexpr (KC) {
    const int row = base + (lane & 31);
    const int chunk = kk * 2 + (lane >> 5);
    return *reinterpret_cast<const bf16x8*>(stage + row * (BK * 2) + ((chunk ^ kc_swz<BK>(row)) << 4));
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

// Position in a workgroup's sequence of k-tiles, in scalar registers: global base addresses of the next
// tile and the number of tiles left in the current run.  A k-slice is at most three runs of consecutive
// tiles (one per segment).  A wave issues one instruction every four cycles and a matrix instruction
// occupies its pipe for 32: seven other instructions fit between two of them for free, and every one
// beyond that is a bubble in the matrix pipe.  The cursor therefore advances without branches, in a few
// scalar and/or/add steps (a conditional expression on the fields compiles to a select of addresses,
// which puts the cursor into memory, or to branches), and the main loop calls the two halves of the
// update in two different gaps.  Past the end of the last run the cursor stays on the last tile: the
// pipeline requests NS - 1 tiles more than it uses, and those refetch valid data.
struct KCursor {
  uint64_t a, b;      // bases of the next tile
  int rem;            // tiles left in the current run, this one included
  uint64_t step_a, step_b;
  // runs after the current one (MULTI only): what to add to a / b at the switch instead of the step
  // (start of that run minus last tile of the one before), and the run lengths (0: no such run)
  uint64_t da1, db1, da2, db2;
  int rn1, rn2;
  // masks of the update in progress: all ones when the run has another tile / when the next run starts
  uint64_t m_stay, m_sw;
};
// first half: hands out the current tile and moves the bases on
template <bool MULTI>
__device__ __forceinline__ void cursor_bases(KCursor& c, const char*& abase, const char*& bbase) {
  abase = (const char*)c.a;
  bbase = (const char*)c.b;
  c.m_stay = (uint64_t)(int64_t)(c.rem > 1 ? -1 : 0);
  if constexpr (MULTI) {
    c.m_sw = (uint64_t)(int64_t)((c.rem <= 1 && c.rn1 > 0) ? -1 : 0);
    c.a += (c.step_a & c.m_stay) | (c.da1 & c.m_sw);
    c.b += (c.step_b & c.m_stay) | (c.db1 & c.m_sw);
  } else {
    c.a += c.step_a & c.m_stay;
    c.b += c.step_b & c.m_stay;
  }
}
// second half: the run counters
template <bool MULTI>
__device__ __forceinline__ void cursor_counts(KCursor& c) {
  const int i_stay = (int)c.m_stay;
  if constexpr (MULTI) {
    const int i_sw = (int)c.m_sw;
    c.rem = ((c.rem - 1) & i_stay) | (c.rn1 & i_sw) | (1 & ~(i_stay | i_sw));
    c.da1 = (c.da2 & c.m_sw) | (c.da1 & ~c.m_sw);
    c.db1 = (c.db2 & c.m_sw) | (c.db1 & ~c.m_sw);
    c.rn1 = (c.rn2 & i_sw) | (c.rn1 & ~i_sw);
    c.rn2 = c.rn2 & ~i_sw;
  } else {
    c.rem += i_stay;  // counts down to 1 and stays there
  }
}
template <bool MULTI>
__device__ __forceinline__ void cursor_next(KCursor& c, const char*& abase, const char*& bbase) {
  cursor_bases<MULTI>(c, abase, bbase);
  cursor_counts<MULTI>(c);
}

// EPI_T: the epilogue kind, plus EPI_DROP when the result passes a dropout site (a separate instantiation,
// so that the kernels without dropout keep their register budget).
constexpr int EPI_DROP = 8;
// ... plus EPI_GROUP for a grouped launch (several problems of one shape, operands from a pointer table).
constexpr int EPI_GROUP = 16;
template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, int EPI_T, int NS, int MINW, int BK>
__global__ __launch_bounds__(WM * WN * 64, MINW) void gemm_mfma_kernel(GemmDesc g, GemmEpi e, int tiles_m,
                                                                int tiles_n, int split_k) {
  constexpr int EPI = EPI_T & (EPI_DROP - 1);
  constexpr bool DROP = (EPI_T & EPI_DROP) != 0;
  constexpr bool GROUP = (EPI_T & EPI_GROUP) != 0;
  constexpr int NW = WM * WN;
  constexpr int TMW = BM / WM, TNW = BN / WN;
  constexpr int MI = TMW / 32, NI = TNW / 32;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
  constexpr int STAGE = A_BYTES + B_BYTES;
  constexpr int A_DMA = A_BYTES / 1024 / NW, B_DMA = B_BYTES / 1024 / NW;  // DMA instructions per wave
  constexpr int DMA_PER_TILE = A_DMA + B_DMA;
  static_assert(A_BYTES % (1024 * NW) == 0 && B_BYTES % (1024 * NW) == 0, "tile vs wave count");
  static_assert((NS - 1) * DMA_PER_TILE < 64, "vmcnt range");
  constexpr int KSTEPS = BK / 16;
  constexpr int RPB = 512 / BK;  // rows of a k-contiguous stage per 1 KB block
  constexpr int CPRK = BK / 8;   // 16-byte chunks per such row
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;

  // ---- XCD-aware mapping.  Workgroup ids are dealt round-robin to the 8 XCDs; give each XCD a
  // contiguous chunk of the (k-slice, tile) space so that whole k-slices, and compact blocks of
  // tiles inside them, share operand panels through one L2.
  const int nb = tiles_m * tiles_n;
  const int ngr = GROUP ? g.ngroups : 1;
  int L;
  {
    const int total = nb * split_k * ngr;
    const int bid = blockIdx.x;
    const int xcd = bid & 7, idx = bid >> 3;
    const int nb8 = (total + 7) >> 3, rem = total & 7;
    if (rem == 0 || xcd < rem) L = xcd * nb8 + idx; else L = rem * nb8 + (xcd - rem) * (nb8 - 1) + idx;
  }
  // grouped launch: the problem this workgroup belongs to, and its operands and outputs
  const void *seg_a = g.seg[0].A, *seg_b = g.seg[0].B;
  void *so0 = e.out0, *so1 = e.out1, *so2 = e.out2;
  if constexpr (GROUP) {
    {
      const int grp = L / (nb * split_k);
      L -= grp * nb * split_k;
      const void* const* t = g.groups + (size_t)grp * GEMM_GROUP_PTRS;
      seg_a = t[0]; seg_b = t[1];
      so0 = const_cast<void*>(t[2]); so1 = const_cast<void*>(t[3]); so2 = const_cast<void*>(t[4]);
    }
  }
  const int ks = L / nb;  // split-k slice
  L -= ks * nb;
  constexpr int GM = 8;
  const int per_group = GM * tiles_n;
  const int group = L / per_group, in_g = L - group * per_group;
  const int first_m = group * GM;
  const int gsz = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
  const int tm = first_m + in_g % gsz, tn = in_g / gsz;
  const int m0 = tm * BM, n0 = tn * BN;

  // ---- k-tile range of this workgroup (flattened over segments; lda/ldb are equal across segments)
  int nk_total = 0;
  for (int s = 0; s < g.nseg; ++s) nk_total += g.seg[s].K / BK;
  const int per = (nk_total + split_k - 1) / split_k;
  const int kt_begin = ks * per;
  const int kt_end = (kt_begin + per) < nk_total ? (kt_begin + per) : nk_total;
  const int nk = kt_end - kt_begin;
  const int lda = g.seg[0].lda, ldb = g.seg[0].ldb;

  // ---- per-lane byte offsets of this wave's DMA slots (loop invariant)
  uint32_t a_off[A_DMA], b_off[B_DMA];
#pragma unroll
  for (int i = 0; i < A_DMA; ++i) {
    const int q = wave + i * NW;  // 1 KB block inside the A stage
    if constexpr (A_KC) {
      const int row = q * RPB + lane / CPRK;
      const int chunk = (lane % CPRK) ^ kc_swz<BK>(row);
      int gr = m0 + row;
      gr = gr < g.M ? gr : g.M - 1;
      a_off[i] = (uint32_t)gr * (uint32_t)lda * 2u + (uint32_t)chunk * 16u;
    } else {
      constexpr int CPR = BM / 8;  // 16-byte chunks per k-row
      const int slot = q * 64 + lane;
      const int krow = slot / CPR, pch = slot % CPR;
      const int gch = (((pch >> 1) ^ ((krow & 3) << 1)) << 1) | (pch & 1);
      int mm = m0 + gch * 8;
      mm = mm < g.M ? mm : g.M - 8;
      a_off[i] = (uint32_t)krow * (uint32_t)lda * 2u + (uint32_t)mm * 2u;
    }
  }
#pragma unroll
  for (int i = 0; i < B_DMA; ++i) {
    const int q = wave + i * NW;
    if constexpr (B_KC) {
      const int row = q * RPB + lane / CPRK;
      const int chunk = (lane % CPRK) ^ kc_swz<BK>(row);
      int gr = n0 + row;
      gr = gr < g.N ? gr : g.N - 1;
      b_off[i] = (uint32_t)gr * (uint32_t)ldb * 2u + (uint32_t)chunk * 16u;
    } else {
      constexpr int CPR = BN / 8;
      const int slot = q * 64 + lane;
      const int krow = slot / CPR, pch = slot % CPR;
      const int gch = (((pch >> 1) ^ ((krow & 3) << 1)) << 1) | (pch & 1);
      int nn = n0 + gch * 8;
      nn = nn < g.N ? nn : g.N - 8;
      b_off[i] = (uint32_t)krow * (uint32_t)ldb * 2u + (uint32_t)nn * 2u;
    }
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)smem;

  KCursor kc;
  kc.step_a = A_KC ? (uint64_t)BK * 2 : (uint64_t)BK * (uint64_t)lda * 2;
  kc.step_b = B_KC ? (uint64_t)BK * 2 : (uint64_t)BK * (uint64_t)ldb * 2;
  kc.da1 = kc.db1 = kc.da2 = kc.db2 = 0;
  kc.rn1 = kc.rn2 = 0;
  kc.m_stay = kc.m_sw = 0;
  if (g.nseg == 1) {
    kc.a = (uint64_t)seg_a + (uint64_t)kt_begin * kc.step_a;
    kc.b = (uint64_t)seg_b + (uint64_t)kt_begin * kc.step_b;
    kc.rem = nk;
  } else {  // several segments are never split along k
    const int n0 = g.seg[0].K / BK, n1 = g.seg[1].K / BK;
    kc.a = (uint64_t)g.seg[0].A; kc.b = (uint64_t)g.seg[0].B; kc.rem = n0;
    kc.da1 = (uint64_t)g.seg[1].A - (kc.a + (uint64_t)(n0 - 1) * kc.step_a);
    kc.db1 = (uint64_t)g.seg[1].B - (kc.b + (uint64_t)(n0 - 1) * kc.step_b);
    kc.rn1 = n1;
    if (g.nseg > 2) {
      kc.da2 = (uint64_t)g.seg[2].A - ((uint64_t)g.seg[1].A + (uint64_t)(n1 - 1) * kc.step_a);
      kc.db2 = (uint64_t)g.seg[2].B - ((uint64_t)g.seg[1].B + (uint64_t)(n1 - 1) * kc.step_b);
      kc.rn2 = g.seg[2].K / BK;
    }
  }
  // Issue DMA instructions [d0, d1) of a k-tile into stage `st`; a tile's DMA_PER_TILE instructions
  // per wave are numbered A slots first, then B slots.
  // The DMA instructions take their base address from scalar registers.  Addresses that came out of a group
  // table are the same in every lane but live in vector registers: broadcast them from the first lane.
  auto uniform = [](const char* q) __attribute__((always_inline)) {
    const uint64_t v = (uint64_t)q;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const char*)(((uint64_t)hi << 32) | lo);
  };
  auto dma_part = [&](const char* abase, const char* bbase, int st, int d0, int d1) __attribute__((always_inline)) {
    // (also without a group table: where the compiler keeps a cursor value in vector registers across a
    // barrier this moves it back; on a value that is already scalar it folds away)
    abase = uniform(abase);
    bbase = uniform(bbase);
    const uint32_t sa = lds0 + st * STAGE, sb = sa + A_BYTES;
#pragma unroll
    for (int d = 0; d < DMA_PER_TILE; ++d) {
      if (d < d0 || d >= d1) continue;
      if (d < A_DMA) dma_1k(sa + (wave + d * NW) * 1024, abase, a_off[d < A_DMA ? d : 0]);
      else dma_1k(sb + (wave + (d - A_DMA) * NW) * 1024, bbase, b_off[d >= A_DMA ? d - A_DMA : 0]);
    }
  };

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  bf16x8 fa[2][MI], fb[2][NI];
  auto load_frags = [&](int st, int kk, int slot) __attribute__((always_inline)) {
    const char* sa = smem + st * STAGE;
    const char* sb = sa + A_BYTES;
#pragma unroll
    for (int i = 0; i < MI; ++i) fa[slot][i] = load_frag<BM, A_KC, BK>(sa, wm * TMW + i * 32, kk, lane);
#pragma unroll
    for (int j = 0; j < NI; ++j) fb[slot][j] = load_frag<BN, B_KC, BK>(sb, wn * TNW + j * 32, kk, lane);
  };
  // One k-step in MI chunks.  Chunk i issues its share of `dcount` DMA instructions (numbers dbase..)
  // of a k-tile into stage dst, fetches its share of the next k-step's fragments (stage ld_st,
  // k-step ld_kk, into register set nxt) and runs the MFMAs of accumulator row i from register set
  // cur.  The DMA instructions are spread out because a wave that issues them back to back sits in
  // the memory pipeline's issue queue instead of feeding the matrix unit.  The fragment reads all go
  // into the first MI - 1 chunks, in the order the next k-step consumes them (its first chunk needs
  // A row 0 and every B column): the last chunk's MFMAs then cover their latency, so that neither the
  // next k-step's first MFMA nor the wait before a barrier finds a read still in flight.
  auto kstep = [&](int cur, int ld_st, int ld_kk, int nxt, const char* abase, const char* bbase, int dst,
                   int dbase, int dcount, auto&& gap) __attribute__((always_inline)) {
    const char* sa = smem + ld_st * STAGE;
    const char* sb = sa + A_BYTES;
    constexpr int NLD = MI + NI;              // fragment reads of one k-step
    constexpr int LCH = MI > 1 ? MI - 1 : 1;  // chunks that carry them
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      if (dcount > 0) dma_part(abase, bbase, dst, dbase + i * dcount / MI, dbase + (i + 1) * dcount / MI);
#pragma unroll
      for (int q = 0; q < NLD; ++q) {  // read q: A row 0, B columns 0 .. NI-1, A rows 1 .. MI-1
        if (q * LCH / NLD != i) continue;
        if (q == 0) fa[nxt][0] = load_frag<BM, A_KC, BK>(sa, wm * TMW, ld_kk, lane);
        else if (q <= NI) fb[nxt][q - 1] = load_frag<BN, B_KC, BK>(sb, wn * TNW + (q - 1) * 32, ld_kk, lane);
        else fa[nxt][q - NI] = load_frag<BM, A_KC, BK>(sa, wm * TMW + (q - NI) * 32, ld_kk, lane);
      }
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
        if (j == 0) gap(i);  // scalar bookkeeping of the caller, in the shadow of the MFMA just issued
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto no_gap = [](int) __attribute__((always_inline)) {};
  constexpr int H0 = DMA_PER_TILE / 2;  // a tile's DMA is issued in two parts: [0, H0) and [H0, DMA_PER_TILE)

  // The k loop, compiled twice: for one run of tiles (one segment) and for several.
  auto k_loop = [&](auto multi_tag) __attribute__((always_inline)) {
    constexpr bool MULTI = decltype(multi_tag)::value;
    // Prologue: fill stages 0 .. NS-2 and the first part of stage NS-1, wait for tile 0.
    const char *ab, *bb;
#pragma unroll
    for (int s = 0; s + 1 < NS; ++s) {
      cursor_next<MULTI>(kc, ab, bb);
      dma_part(ab, bb, s, 0, DMA_PER_TILE);
    }
    cursor_next<MULTI>(kc, ab, bb);
    dma_part(ab, bb, NS - 1, 0, H0);
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((NS - 2) * DMA_PER_TILE + H0) : "memory");
    load_frags(0, 0, 0);
    // One k-tile out of stage s.  k-step 0 also issues the second part of tile t+NS-1 (its stage was
    // released at the previous barrier) and, in two of its gaps, works out the addresses of tile t+NS:
    // whatever stands between the barrier and the next MFMA is a bubble in the matrix pipe.  k-steps
    // 1 .. KSTEPS-2 issue nothing.  At the barrier tile t+1 has landed (this wave's part) and all of
    // this wave's reads of stage s are done; after it that holds for every wave, so the last k-step
    // refills stage s with the first part of tile t+NS.
    auto ktile = [&](int s) __attribute__((always_inline)) {
      const char *an = ab, *bn = bb;
      kstep(0, s, 1, 1, ab, bb, (s + NS - 1) % NS, H0, DMA_PER_TILE - H0, [&](int i) __attribute__((always_inline)) {
        if (i == 0) cursor_bases<MULTI>(kc, an, bn);
        if (i == 1) cursor_counts<MULTI>(kc);
      });
#pragma unroll
      for (int kk = 1; kk + 1 < KSTEPS; ++kk) kstep(kk & 1, s, kk + 1, (kk + 1) & 1, ab, bb, 0, 0, 0, no_gap);
      ab = an; bb = bn;  // tile t + NS
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"((NS - 2) * DMA_PER_TILE) : "memory");
      kstep((KSTEPS - 1) & 1, (s + 1) % NS, 0, 0, ab, bb, s, 0, H0, no_gap);
    };
    // whole rounds of the stage ring run without a test per tile; the last, partial round tests
    int t = 0;
    for (; t + NS <= nk; t += NS) {
#pragma unroll
      for (int s = 0; s < NS; ++s) ktile(s);
    }
#pragma unroll
    for (int s = 0; s + 1 < NS; ++s)
      if (t + s < nk) ktile(s);
    // drain DMA that was issued past the end before LDS is released
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  };
  if (nk > 0) {
    if (g.nseg == 1) k_loop(std::false_type{});
    else k_loop(std::true_type{});
  }

  // Output placement of the epilogue, in locals: the reproducible split reduction redirects it.  There this
  // k-slice stores its partial sums, as a plain M x N float32 matrix of its own, instead of adding them into the
  // output; splitk_reduce_kernel adds the slices up afterwards.
  int ep_ld0 = e.ld0, ep_split_n = e.split_n, ep_acc = e.accumulate, ep_sk = split_k;
  if constexpr (EPI == EPI_SPLIT_F32 && !GROUP) {
    if (e.aux0 != nullptr && split_k > 1) {
      so0 = (float*)const_cast<void*>(e.aux0) + (size_t)ks * (size_t)g.M * (size_t)g.N;
      ep_ld0 = g.N;
      ep_split_n = 1 << 30;
      ep_acc = 0;
      ep_sk = 1;
    }
  }
  // ---- epilogue.  acc[i][j][r]: row = (r/4)*8 + (lane/32)*4 + r%4, col = lane%32 of the 32x32 tile.
  // Interior wave tiles (the common case) are transposed through LDS, 64 rows at a time, so that
  // each lane ends up with 4 consecutive columns of one row: auxiliary loads and the stores are
  // then 8- or 16-byte vector accesses covering whole rows of the wave tile.  Edge tiles take the
  // predicated per-element path further down.
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");  // every wave is done with the k-loop stages
  {
    constexpr int EP_LD = TNW + 8;  // floats per staged row
    const int mw = m0 + wm * TMW, nw = n0 + wn * TNW;
    bool interior = (mw + TMW <= g.M) && (nw + TNW <= g.N) && (ep_ld0 % 8 == 0) && (e.ld_aux % 8 == 0);
    if constexpr (EPI == EPI_SPLIT_F32)
      interior = interior && (nw / ep_split_n == (nw + TNW - 1) / ep_split_n) && (ep_split_n % 4 == 0);
    if constexpr (EPI == EPI_SPLIT_F32) {
      // split-k partial sums go out as float atomics straight from the accumulator registers
      // (32 consecutive floats per half-wave and row)
      if (interior && ep_sk > 1) {
        const int cl = lane & 31, rl = (lane >> 5) << 2;
        const int which = nw / ep_split_n;
        float* dst0 = (float*)(which == 0 ? so0 : which == 1 ? so1 : so2) + (nw - which * ep_split_n) + cl;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float* rowp = dst0 + (size_t)(mw + i * 32 + ((r >> 2) << 3) + rl + (r & 3)) * ep_ld0;
#pragma unroll
            for (int j = 0; j < NI; ++j) unsafeAtomicAdd(rowp + j * 32, acc[i][j][r]);
          }
        return;
      }
    }
    if (interior) {
      float* stg = reinterpret_cast<float*>(smem) + wave * (64 * EP_LD);
      const int cl = lane & 31, rl = (lane >> 5) << 2;
      // 64 rows of the wave tile into the staging block (a macro, so that the textually included copies of the
      // row-wise epilogue below can use it as well)
#define T5MI_STAGE_HALF(half)                                                                              \
  do {                                                                                                     \
    _Pragma("unroll") for (int ii = 0; ii < 2; ++ii)                                                       \
      _Pragma("unroll") for (int j = 0; j < NI; ++j)                                                       \
        _Pragma("unroll") for (int r = 0; r < 16; ++r)                                                     \
          stg[(ii * 32 + ((r >> 2) << 3) + rl + (r & 3)) * EP_LD + j * 32 + cl] = acc[(half) * 2 + ii][j][r]; \
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                                                     \
    __builtin_amdgcn_wave_barrier();                                                                       \
  } while (0)
      if constexpr (EPI == EPI_GEGLU_FWD) {
        // The activation is chosen once per tile, outside the element loops: tested per element, the choice
        // becomes a branch around every evaluation and the epilogue falls apart into hundreds of short blocks.
        auto passes = [&](auto erf_tag) __attribute__((always_inline)) {
        constexpr bool ERF = decltype(erf_tag)::value;
#pragma unroll
        for (int half = 0; half < MI / 2; ++half) {
          T5MI_STAGE_HALF(half);
          const int mh = mw + half * 64;
          // staged columns: [u 32 | w 32] pairs; lane takes 4 consecutive f of one row
          constexpr int LPR = TNW / 8;  // lanes per row
          const int fl = (lane % LPR) * 4;
          const int pc = (fl >> 5) * 64 + (fl & 31);  // staged column of u; w is 32 further
          const int f = (nw >> 1) + fl;
#pragma unroll
          for (int it = 0; it < 64 / (64 / LPR); ++it) {
            const int rloc = it * (64 / LPR) + lane / LPR;
            const f32x4 uu = *reinterpret_cast<const f32x4*>(stg + rloc * EP_LD + pc);
            const f32x4 ww = *reinterpret_cast<const f32x4*>(stg + rloc * EP_LD + pc + 32);
            bf16x4 gpb, glb, ab;
            f32x4 mk = {1.f, 1.f, 1.f, 1.f};
            if constexpr (DROP) {
              const uint32_t k1 = drop_row_key(e.drop, (uint32_t)(mh + rloc));
#pragma unroll
              for (int q = 0; q < 4; ++q) mk[q] = drop_mult(e.drop, k1, (uint32_t)(f + q));
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              float gl, dgl;
              if constexpr (ERF) gelu_erf_both(uu[q], gl, dgl); else gelu_tanh_both(uu[q], gl, dgl);
              gpb[q] = (bf16)(ww[q] * dgl * mk[q]);
              glb[q] = (bf16)(gl * mk[q]);
              ab[q] = (bf16)(gl * ww[q] * mk[q]);
            }
            const size_t o = (size_t)(mh + rloc) * ep_ld0 + f;
            st_stream(reinterpret_cast<bf16x4*>((bf16*)e.out0 + o), gpb);
            st_stream(reinterpret_cast<bf16x4*>((bf16*)e.out1 + o), glb);
            st_stream(reinterpret_cast<bf16x4*>((bf16*)e.out2 + o), ab);
          }
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          __builtin_amdgcn_wave_barrier();
        }
        };
        if (e.act == ACT_GELU_ERF) passes(std::true_type{}); else passes(std::false_type{});
      } else {
        // Run-time properties of the epilogue (operand and output types, the rarely used ReLU forms, accumulation)
        // are turned into compile-time ones here, once per tile: tested where they are used, inside the unrolled
        // element loops, each becomes a branch per instruction and the epilogue falls apart into short blocks that
        // the scheduler cannot overlap (gated-GELU forward +13 %, output projection with the float32 residual +5 %).
        // The rare combinations share one copy that reads them at run time, so that the number of copies stays small.
        if constexpr (EPI == EPI_GEGLU_BWD) {
#define T5MI_EPI_AF 0
#define T5MI_EPI_OB 1
#define T5MI_EPI_SP 0
#include "gemm_epilogue_rows.inc"
#undef T5MI_EPI_AF
#undef T5MI_EPI_OB
#undef T5MI_EPI_SP
        } else if constexpr (EPI == EPI_SPLIT_F32) {
#define T5MI_EPI_AF 0
#define T5MI_EPI_OB 0
#define T5MI_EPI_SP 2
#include "gemm_epilogue_rows.inc"
#undef T5MI_EPI_AF
#undef T5MI_EPI_OB
#undef T5MI_EPI_SP
        } else if constexpr (EPI == EPI_RESID) {
          const bool af = e.aux_type != IN_BF16;
          const bool ob = e.out_type == IN_BF16;
          if (e.aux_mask != 0) {
#define T5MI_EPI_AF 2
#define T5MI_EPI_OB 2
#define T5MI_EPI_SP 1
#include "gemm_epilogue_rows.inc"
#undef T5MI_EPI_AF
#undef T5MI_EPI_OB
#undef T5MI_EPI_SP
          } else if (af) {
            if (ob) {
#define T5MI_EPI_AF 1
#define T5MI_EPI_OB 1
#define T5MI_EPI_SP 0
#include "gemm_epilogue_rows.inc"
#undef T5MI_EPI_AF
#undef T5MI_EPI_OB
#undef T5MI_EPI_SP
            } else {
#define T5MI_EPI_AF 1
#define T5MI_EPI_OB 0
#define T5MI_EPI_SP 0
#include "gemm_epilogue_rows.inc"
#undef T5MI_EPI_AF
#undef T5MI_EPI_OB
#undef T5MI_EPI_SP
            }
          } else {
            if (ob) {
#define T5MI_EPI_AF 0
#define T5MI_EPI_OB 1
#define T5MI_EPI_SP 0
#include "gemm_epilogue_rows.inc"
#undef T5MI_EPI_AF
#undef T5MI_EPI_OB
#undef T5MI_EPI_SP
            } else {
#define T5MI_EPI_AF 0
#define T5MI_EPI_OB 0
#define T5MI_EPI_SP 0
#include "gemm_epilogue_rows.inc"
#undef T5MI_EPI_AF
#undef T5MI_EPI_OB
#undef T5MI_EPI_SP
            }
          }
        } else {
          // plain store
          if (e.act == ACT_RELU) {
#define T5MI_EPI_AF 0
#define T5MI_EPI_OB 2
#define T5MI_EPI_SP 1
#include "gemm_epilogue_rows.inc"
#undef T5MI_EPI_AF
#undef T5MI_EPI_OB
#undef T5MI_EPI_SP
          } else if (e.out_type == IN_BF16) {
#define T5MI_EPI_AF 0
#define T5MI_EPI_OB 1
#define T5MI_EPI_SP 0
#include "gemm_epilogue_rows.inc"
#undef T5MI_EPI_AF
#undef T5MI_EPI_OB
#undef T5MI_EPI_SP
          } else {
#define T5MI_EPI_AF 0
#define T5MI_EPI_OB 0
#define T5MI_EPI_SP 0
#include "gemm_epilogue_rows.inc"
#undef T5MI_EPI_AF
#undef T5MI_EPI_OB
#undef T5MI_EPI_SP
          }
        }
      }
      return;
    }
  }
  // ---- edge tiles: per-element bounds checks
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
          const float uu = acc[i][j][r], ww = acc[i][j + 1][r];
          float gl, dgl;
          gelu_both(e.act, uu, gl, dgl);
          const size_t o = (size_t)m * ep_ld0 + f;
          const float mk = DROP ? drop_mult(e.drop, drop_row_key(e.drop, (uint32_t)m), (uint32_t)f) : 1.f;
          ((bf16*)e.out0)[o] = (bf16)(ww * dgl * mk);
          ((bf16*)e.out1)[o] = (bf16)(gl * mk);
          ((bf16*)e.out2)[o] = (bf16)(gl * ww * mk);
        }
      } else {
#pragma unroll
        for (int j = 0; j < NI; ++j) {
          const int n = n0 + wn * TNW + j * 32 + col_l;
          if (n >= g.N) continue;
          float v = acc[i][j][r];
          const size_t o = (size_t)m * ep_ld0 + n;
          float mk = 1.f;
          if constexpr (EPI == EPI_STORE || EPI == EPI_RESID)
            if constexpr (DROP) mk = drop_mult(e.drop, drop_row_key(e.drop, (uint32_t)m), (uint32_t)n);
          if constexpr (EPI == EPI_STORE) {
            if (e.act == ACT_RELU) v = fmaxf(v, 0.f);
            v *= mk;
            if (e.out_type == IN_BF16) ((bf16*)e.out0)[o] = (bf16)v; else ((float*)e.out0)[o] = v;
          } else if constexpr (EPI == EPI_RESID) {
            const size_t oa = (size_t)m * (e.ld_aux ? e.ld_aux : ep_ld0) + n;
            const float a = e.aux_type == IN_BF16 ? (float)((const bf16*)e.aux0)[oa] : ((const float*)e.aux0)[oa];
            const float r = e.aux_mask ? (a > 0.f ? v * (DROP ? e.drop.scale : 1.f) : 0.f) : fmaf(v, mk, a);
            if (e.out_type == IN_BF16) ((bf16*)e.out0)[o] = (bf16)r; else ((float*)e.out0)[o] = r;
          } else if constexpr (EPI == EPI_GEGLU_BWD) {
            const size_t oa = (size_t)m * (e.ld_aux ? e.ld_aux : ep_ld0) + n;
            const float gp = (float)((const bf16*)e.aux0)[oa], gl = (float)((const bf16*)e.aux1)[oa];
            ((bf16*)e.out0)[o] = (bf16)(v * gp);
            ((bf16*)e.out1)[o] = (bf16)(v * gl);
          } else {  // EPI_SPLIT_F32
            const int which = n / ep_split_n, nn = n - which * ep_split_n;
            float* dst = (float*)(which == 0 ? so0 : which == 1 ? so1 : so2) + (size_t)m * ep_ld0 + nn;
            if (ep_sk > 1) unsafeAtomicAdd(dst, v);
            else *dst = ep_acc ? *dst + v : v;
          }
        }
      }
    }
  }
}

struct PtrChunk { const void* p[64]; };
__global__ void fill_ptrs_kernel(PtrChunk c, int n, const void** dst) {
  if ((int)threadIdx.x < n) dst[threadIdx.x] = c.p[threadIdx.x];
}

__global__ void zero_split_kernel(GemmEpi e, int M, int N) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)M * N) return;
  const int m = (int)(idx / N), n = (int)(idx % N);
  const int which = n / e.split_n, nn = n - which * e.split_n;
  float* dst = (float*)(which == 0 ? e.out0 : which == 1 ? e.out1 : e.out2);
  dst[(size_t)m * e.ld0 + nn] = 0.f;
}

// out[m][n] (+)= partials[0][m][n] + partials[1][m][n] + ... in that order; out as in EPI_SPLIT_F32.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmEpi e, int M, int N, int slices) {
  const int64_t idx = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;  // N % 4 == 0 (checked by the launcher)
  if (idx >= (int64_t)M * N) return;
  const size_t mn = (size_t)M * N;
  const float* partials = (const float*)e.aux0;
  f32x4 acc = *reinterpret_cast<const f32x4*>(partials + idx);
  for (int s = 1; s < slices; ++s) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(partials + (size_t)s * mn + idx);
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] += v[q];
  }
  const int m = (int)(idx / N), n = (int)(idx % N);
  const int which = n / e.split_n, nn = n - which * e.split_n;  // split_n % 4 == 0: the four columns share an output
  float* dst = (float*)(which == 0 ? e.out0 : which == 1 ? e.out1 : e.out2) + (size_t)m * e.ld0 + nn;
  if (e.accumulate) {
    const f32x4 old = *reinterpret_cast<const f32x4*>(dst);
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] += old[q];
  }
  *reinterpret_cast<f32x4*>(dst) = acc;
}

// Tile size and k split of a weight-gradient GEMM (EPI_SPLIT_F32): few output tiles, very long k.
// Small outputs take 128x128 tiles (fewer k-slices, hence fewer partial sums per output element); k is split
// so that the workgroups fill whole rounds of the 256 compute units.
void wgrad_plan(const GemmDesc& g, const GemmEpi& e, int ngr, bool& big, int& split_k) {
  int nk = 0;
  for (int s = 0; s < g.nseg; ++s) nk += g.seg[s].K / KQ;
  const int64_t t256 = (int64_t)ceil_div(g.M, 256) * ceil_div(g.N, 256) * ngr;
  const int64_t t128 = (int64_t)ceil_div(g.M, 128) * ceil_div(g.N, 128) * ngr;
  // 256x256 tiles from 48 output tiles on, and from 24 when the reduction is long (measured at d_model 768:
  // dWi 3x16 tiles -18 % at 65536 and -10 % at 16384 tokens; dWo_ff 8x3 and dWqkv 3x9 tiles -14 % at 65536
  // tokens but +10..18 % at 16384, where a workgroup's share of k no longer pays for the larger epilogue)
  big = t256 >= 48 || (t256 >= 24 && nk * KQ >= 49152);
  // grouped small outputs (12 x 768 x 768: 432 tiles of 128x128): one round of small tiles over the whole
  // reduction, no split and no atomics, beats 256x256 tiles split seven ways (0.20 -> 0.17 ms at 4096 tokens)
  if (ngr > 1 && t128 <= 512) big = false;
  const int64_t tiles = big ? t256 : t128;
  const int per_cu = big ? 1 : 2;  // concurrent workgroups per compute unit (LDS-limited)
  double best = -1.0;
  split_k = 1;
  for (int sp = 1; sp <= 32; ++sp) {
    if (sp > 1 && nk / sp < 8) break;
    const int64_t wgs = tiles * sp, slots = 256 * per_cu;
    const int64_t rounds = (wgs + slots - 1) / slots;
    double eff;
    if (big) {
      // time = rounds x (a workgroup's k-tiles + its epilogue); the epilogue of a 256x256 slice (65536 float
      // atomics beside those of 255 other workgroups) costs about as much as 12 k-tiles of 64 (measured)
      eff = 1.0 / ((double)rounds * ((double)nk / sp + 12.0));
    } else {
      eff = (double)wgs / (double)(rounds * slots) - 0.012 * sp;
    }
    if (eff > best) { best = eff; split_k = sp; }
  }
  (void)e;
}
// whether the reproducible two-pass reduction applies to this problem
bool split_partials_ok(const GemmDesc& g, const GemmEpi& e) {
  return e.aux0 != nullptr && g.ngroups <= 1 && g.N % 4 == 0 && e.split_n % 4 == 0 && e.ld0 % 4 == 0;
}

template <int BM, int BN, int WM, int WN, bool A_KC, bool B_KC, int EPI, int NS = 4, int MINW = 1, int BK = 32>
hipError_t launch_cfg(const GemmDesc& g, const GemmEpi& e, int split_k, hipStream_t st) {
  auto kern = gemm_mfma_kernel<BM, BN, WM, WN, A_KC, B_KC, EPI, NS, MINW, BK>;
  constexpr int lds_loop = NS * (BM + BN) * BK * 2;
  constexpr int lds_epi = WM * WN * 64 * (BN / WN + 8) * 4;
  constexpr int lds = lds_loop > lds_epi ? lds_loop : lds_epi;
  // once per instantiation; setting it twice is harmless, so a relaxed flag is enough
  static std::atomic<bool> attr_set{false};
  if (!attr_set.load(std::memory_order_relaxed)) {
    hipError_t err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (err != hipSuccess) return err;
    attr_set.store(true, std::memory_order_relaxed);
  }
  const int tiles_m = ceil_div(g.M, BM), tiles_n = ceil_div(g.N, BN);
  const int ngr = (EPI & EPI_GROUP) ? g.ngroups : 1;
  kern<<<tiles_m * tiles_n * split_k * ngr, WM * WN * 64, lds, st>>>(g, e, tiles_m, tiles_n, split_k);
  return hipGetLastError();
}

template <bool A_KC, bool B_KC, int EPI_T>
hipError_t launch_layout(const GemmDesc& g, const GemmEpi& e, hipStream_t st) {
  constexpr int EPI = EPI_T & (EPI_DROP - 1);
  int nk = 0;
  for (int s = 0; s < g.nseg; ++s) nk += g.seg[s].K / KQ;
  // a grouped launch (weight gradients of several layers) counts the tiles of all its problems
  const int ngr = (EPI_T & EPI_GROUP) ? g.ngroups : 1;
  const int64_t t256 = (int64_t)ceil_div(g.M, 256) * ceil_div(g.N, 256) * ngr;
  const int64_t t128 = (int64_t)ceil_div(g.M, 128) * ceil_div(g.N, 128) * ngr;
  bool big = t256 >= 192;
  int split_k = 1;
  bool two_pass = false;  // reproducible split reduction through the partial-sum buffer in GemmEpi::aux0
  if constexpr (EPI == EPI_SPLIT_F32) {
    // Partial sums of the k-slices meet in float32 atomics on a zeroed output, or, when the caller provides
    // room for them, in a second pass that adds them up in a fixed order.
    wgrad_plan(g, e, ngr, big, split_k);
    if (ngr > 1 && !e.accumulate) return hipErrorInvalidValue;  // grouped outputs are cleared by the caller
    two_pass = split_k > 1 && split_partials_ok(g, e);
    if (split_k > 1 && !e.accumulate && !two_pass) {
      zero_split_kernel<<<ceil_div((int64_t)g.M * g.N, 256), 256, 0, st>>>(e, g.M, g.N);
      hipError_t err = hipGetLastError();
      if (err != hipSuccess) return err;
    }
  }
  GemmEpi ee = e;
  if constexpr (EPI == EPI_SPLIT_F32) {
    if (!two_pass) ee.aux0 = nullptr;
  }
  auto finish = [&](hipError_t err) {
    if (err != hipSuccess || !two_pass) return err;
    splitk_reduce_kernel<<<ceil_div((int64_t)g.M * g.N / 4, 256), 256, 0, st>>>(ee, g.M, g.N, split_k);
    return hipGetLastError();
  };
  if constexpr (EPI == EPI_SPLIT_F32) {
    if (big) return finish(launch_cfg<256, 256, 2, 2, A_KC, B_KC, EPI_T, 5, 1>(g, ee, split_k, st));
    return finish(launch_cfg<128, 128, 2, 2, A_KC, B_KC, EPI_T, 4, 1>(g, ee, split_k, st));
  }
  if (big) {
    // short k loops: two 256x128 workgroups per compute unit hide each other's prologue/epilogue
    // and so do the epilogue-heavy gated-GELU kernels (three outputs, or two inputs and two outputs);
    // the gated-GELU forward goes back to one 256x256 tile once k is long enough (measured: better
    // from K = 768, worse at K = 512) because the smaller tiles re-stream more operand data
    // residual epilogues into a narrow output (N < 1024: T5.1.1-Small/Base widths), measured per shape:
    // K <= 512 as below (256x128), 128x128 tiles for K up to 768 (-6..15 % at N = 768), 256x256 beyond
    // (-4..9 %)
    if (EPI_T == EPI_RESID && g.N < 1024 && nk > 8) {
      if (nk <= 12) return launch_cfg<128, 128, 2, 2, A_KC, B_KC, EPI_T, 4, 1>(g, e, split_k, st);
      if constexpr (A_KC) return launch_cfg<256, 256, 2, 2, A_KC, B_KC, EPI_T, 2, 1, 64>(g, e, split_k, st);
      return launch_cfg<256, 256, 2, 2, A_KC, B_KC, EPI_T, 5, 1>(g, e, split_k, st);
    }
    // the residual epilogue with dropout does not fit the 256x256 tile's register budget (it would spill)
    if (EPI_T == (EPI_RESID | EPI_DROP)) return launch_cfg<256, 128, 2, 2, A_KC, B_KC, EPI_T, 3, 2>(g, e, split_k, st);
    // (thresholds in units of 64 along k, measured per epilogue: plain stores and the gated-GELU forward gain
    // 10-12 % from the 256x256 tile at K = 768 and lose 7-20 % at K = 512; the residual epilogue is indifferent
    // up to K = 2048)
    if (EPI != EPI_SPLIT_F32 && (((EPI == EPI_STORE || EPI == EPI_GEGLU_FWD) && nk < 12) || EPI == EPI_GEGLU_BWD ||
                                 (EPI == EPI_RESID && nk <= 32)))
      return launch_cfg<256, 128, 2, 2, A_KC, B_KC, EPI_T, 3, 2>(g, e, split_k, st);
    // k-contiguous operands: k-tiles of 64 in two stages.  A DMA instruction then covers eight whole 128-byte
    // rows instead of sixteen half rows (the L1 processes a line per request whatever part of it is used, and
    // at 64 bytes per row that path, not the matrix unit, sets the pace), and there is one barrier per 64 MFMAs
    // instead of per 32.  Measured on the T5.1.1-XL GEMMs against five stages of 32: +7 to +12 %, once a tile's
    // sixteen DMA instructions per wave are issued two per chunk over two k-steps instead of four per chunk over
    // one (issued four at a time they stall the wave in the memory pipeline's queue and the gain is lost).
    // The weight-gradient GEMMs (rows of 512 bytes already) and the 256x128 two-workgroup configuration lose
    // with k-tiles of 64 (-4 % and -25 %) and keep 32.
    if constexpr (A_KC) return launch_cfg<256, 256, 2, 2, A_KC, B_KC, EPI_T, 2, 1, 64>(g, e, split_k, st);
    return launch_cfg<256, 256, 2, 2, A_KC, B_KC, EPI_T, 5, 1>(g, e, split_k, st);
  }
  // too few 256x256 tiles to fill the chip, but a long reduction: 256x128 tiles, two per compute unit
  // (8192 x 768 x 32128: -11 % against 128x128)
  if (EPI != EPI_SPLIT_F32 && t256 >= 64 && nk >= 64)
    return launch_cfg<256, 128, 2, 2, A_KC, B_KC, EPI_T, 3, 2>(g, e, split_k, st);
  return launch_cfg<128, 128, 2, 2, A_KC, B_KC, EPI_T, 4, 1>(g, e, split_k, st);
}

}  // namespace

bool gemm_mfma_supported(const GemmDesc& g, const GemmEpi& e) {
  if (g.in_type != IN_BF16) return false;
  if (g.nseg < 1 || g.nseg > 3) return false;
  if (g.a_kc != g.b_kc) return false;  // implemented: both k-contiguous, or both m/n-contiguous
  for (int s = 0; s < g.nseg; ++s) {
    const GemmSeg& sg = g.seg[s];
    if (sg.K < KQ || sg.K % KQ != 0 || sg.lda % 8 != 0 || sg.ldb % 8 != 0) return false;
    if (sg.lda != g.seg[0].lda || sg.ldb != g.seg[0].ldb) return false;
    if (((uintptr_t)sg.A | (uintptr_t)sg.B) & 15) return false;
  }
  if (g.M < 8 || g.N < 8) return false;
  // per-lane byte offsets are 32-bit
  if ((uint64_t)(g.a_kc ? g.M : KQ) * g.seg[0].lda * 2 >= (1ull << 32)) return false;
  if ((uint64_t)(g.b_kc ? g.N : KQ) * g.seg[0].ldb * 2 >= (1ull << 32)) return false;
  if (!g.a_kc && (g.M % 8 != 0 || g.N % 8 != 0)) return false;
  switch (e.kind) {
    case EPI_STORE: case EPI_RESID: case EPI_GEGLU_BWD:
      return g.a_kc == 1;
    case EPI_GEGLU_FWD:
      return g.a_kc == 1 && g.N % 64 == 0 && e.out_type == IN_BF16;
    case EPI_SPLIT_F32:
      if (g.ngroups > 1 && (!g.groups || !e.accumulate)) return false;
      return g.a_kc == 0 && g.nseg == 1;  // k may be split into slices: one segment only
    default:
      return false;
  }
}

size_t gemm_split_partials_bytes(const GemmDesc& g, const GemmEpi& e) {
  if (e.kind != EPI_SPLIT_F32 || g.ngroups > 1) return 0;
  bool big;
  int split_k;
  wgrad_plan(g, e, 1, big, split_k);
  return split_k > 1 ? (size_t)split_k * (size_t)g.M * (size_t)g.N * sizeof(float) : 0;
}

hipError_t launch_fill_ptrs(const void* const* ptrs, int n, const void** dst, hipStream_t st) {
  for (int i0 = 0; i0 < n; i0 += 64) {
    PtrChunk c;
    const int m = n - i0 < 64 ? n - i0 : 64;
    for (int i = 0; i < 64; ++i) c.p[i] = i < m ? ptrs[i0 + i] : nullptr;
    fill_ptrs_kernel<<<1, 64, 0, st>>>(c, m, dst + i0);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
  return hipSuccess;
}

hipError_t launch_gemm_mfma(const GemmDesc& g, const GemmEpi& e, hipStream_t st) {
  switch (e.kind) {
    case EPI_STORE:
      return e.drop.on ? launch_layout<true, true, EPI_STORE | EPI_DROP>(g, e, st)
                       : launch_layout<true, true, EPI_STORE>(g, e, st);
    case EPI_RESID:
      return e.drop.on ? launch_layout<true, true, EPI_RESID | EPI_DROP>(g, e, st)
                       : launch_layout<true, true, EPI_RESID>(g, e, st);
    case EPI_GEGLU_FWD:
      return e.drop.on ? launch_layout<true, true, EPI_GEGLU_FWD | EPI_DROP>(g, e, st)
                       : launch_layout<true, true, EPI_GEGLU_FWD>(g, e, st);
    case EPI_GEGLU_BWD: return launch_layout<true, true, EPI_GEGLU_BWD>(g, e, st);
    case EPI_SPLIT_F32:
      return g.ngroups > 1 ? launch_layout<false, false, EPI_SPLIT_F32 | EPI_GROUP>(g, e, st)
                           : launch_layout<false, false, EPI_SPLIT_F32>(g, e, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace t5mi
