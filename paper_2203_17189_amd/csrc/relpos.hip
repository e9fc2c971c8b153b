// Relative-position buckets of T5 (the attention bias of the models in paper Sec. 4):
// exact-integer threshold table on the host, lookup kernels on the device.
#include <vector>
#include "kernels.h"

namespace t5mi {

namespace {
// Minimal unsigned big integer (little-endian 32-bit limbs): enough for n^L * E^K comparisons.
struct BigU {
  std::vector<uint32_t> v;
  explicit BigU(uint32_t x = 0) { v.push_back(x); }
  void mul(uint32_t m) {
    uint64_t carry = 0;
    for (size_t i = 0; i < v.size(); ++i) {
      uint64_t t = (uint64_t)v[i] * m + carry;
      v[i] = (uint32_t)t;
      carry = t >> 32;
    }
    if (carry) v.push_back((uint32_t)carry);
  }
  void mul_pow(uint32_t base, int e) {
    for (int i = 0; i < e; ++i) mul(base);
  }
  size_t len() const {
    size_t n = v.size();
    while (n > 1 && v[n - 1] == 0) --n;
    return n;
  }
  // *this >= o
  bool ge(const BigU& o) const {
    size_t a = len(), b = o.len();
    if (a != b) return a > b;
    for (size_t i = a; i-- > 0;) {
      if (v[i] != o.v[i]) return v[i] > o.v[i];
    }
    return true;
  }
};

// (n/E)^L >= (D/E)^m   <=>   n^L * E^m >= D^m * E^L
bool log_index_at_least(int n, int m, int E, int L, int D) {
  BigU lhs(1), rhs(1);
  lhs.mul_pow((uint32_t)n, L);
  lhs.mul_pow((uint32_t)E, m);
  rhs.mul_pow((uint32_t)D, m);
  rhs.mul_pow((uint32_t)E, L);
  return lhs.ge(rhs);
}
}  // namespace

int relpos_build_lut(int bidirectional, int num_buckets, int max_distance, RelposLut* lut) {
  if (num_buckets < 2) return T5_ERR_SHAPE;
  if (bidirectional && (num_buckets % 2 != 0 || num_buckets < 4)) return T5_ERR_SHAPE;
  const int n_side = bidirectional ? num_buckets / 2 : num_buckets;
  const int E = n_side / 2;
  if (E < 1 || max_distance <= E) return T5_ERR_SHAPE;
  const int L = n_side - E;
  const int n_thr = n_side - 1 - E;  // logarithmic indices 1 .. n_thr are distinguishable
  if (n_thr > 64) return T5_ERR_UNSUPPORTED;
  lut->bidirectional = bidirectional ? 1 : 0;
  lut->n_side = n_side;
  lut->max_exact = E;
  lut->n_thr = n_thr;
  for (int i = 0; i < 64; ++i) lut->thr[i] = INT32_MAX;
  int lo_start = E;
  for (int m = 1; m <= n_thr; ++m) {
    // smallest n in [lo_start, max_distance] with index >= m (n = max_distance always qualifies
    // because m <= L - 1 < L)
    int lo = lo_start, hi = max_distance;
    while (lo < hi) {
      int mid = lo + (hi - lo) / 2;
      if (log_index_at_least(mid, m, E, L, max_distance)) hi = mid; else lo = mid + 1;
    }
    lut->thr[m - 1] = lo;
    lo_start = lo;
  }
  return T5_OK;
}

__global__ void relpos_bucket_kernel(const int32_t* __restrict__ rp, int32_t* __restrict__ out, int64_t n,
                                     RelposLut lut) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) out[i] = relpos_bucket_dev(rp[i], lut);
}

hipError_t launch_relpos_bucket(const int32_t* rel_pos, int32_t* out, int64_t n, const RelposLut& lut,
                                hipStream_t st) {
  if (n == 0) return hipSuccess;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  relpos_bucket_kernel<<<(int)blocks, 256, 0, st>>>(rel_pos, out, n, lut);
  return hipGetLastError();
}

template <typename T>
__global__ void relpos_diag_kernel(const T* __restrict__ table, float* __restrict__ diag, int S, int H,
                                   RelposLut lut) {
  const int w = 2 * S - 1;
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= w) return;
  const int b = relpos_bucket_dev(idx - (S - 1), lut);
  for (int h = 0; h < H; ++h) diag[(size_t)h * w + idx] = to_f32(table[b * H + h]);
}

hipError_t launch_relpos_diag(const void* table, int dtype, float* diag, int S, int H, const RelposLut& lut,
                              hipStream_t st) {
  const int w = 2 * S - 1;
  dim3 grid((w + 255) / 256);
  if (dtype == T5_BF16)
    relpos_diag_kernel<bf16><<<grid, 256, 0, st>>>((const bf16*)table, diag, S, H, lut);
  else
    relpos_diag_kernel<float><<<grid, 256, 0, st>>>((const float*)table, diag, S, H, lut);
  return hipGetLastError();
}

// One wave per (bucket c, head h).  Buckets are contiguous distance ranges on each side, so the
// wave sums ddiag over its range in a fixed order (deterministic).
__global__ void relpos_diag_bwd_kernel(const float* __restrict__ ddiag, float* __restrict__ dtable, int S,
                                       int H, int num_buckets, RelposLut lut, int accumulate) {
  const int c = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  const int w = 2 * S - 1;
  int side = 0, cl = c;
  if (lut.bidirectional && c >= lut.n_side) { side = 1; cl = c - lut.n_side; }
  int n_lo, n_hi;  // inclusive distance range of this bucket
  if (cl < lut.max_exact) {
    n_lo = n_hi = cl;
  } else {
    const int k = cl - lut.max_exact;  // logarithmic index
    n_lo = (k == 0) ? lut.max_exact : lut.thr[k - 1];
    n_hi = (cl == lut.n_side - 1) ? (S - 1) : (lut.thr[k] - 1);
  }
  if (n_hi > S - 1) n_hi = S - 1;
  if (side == 1 && n_lo == 0) n_lo = 1;  // distance 0 belongs to the non-positive side
  float s = 0.f;
  for (int n = n_lo + lane; n <= n_hi; n += kWave) {
    const int delta = side ? n : -n;
    s += ddiag[(size_t)h * w + delta + (S - 1)];
  }
  s = wave_sum(s);
  if (lane == 0) {
    float* o = dtable + c * H + h;
    *o = accumulate ? (*o + s) : s;
  }
}

hipError_t launch_relpos_diag_bwd(const float* ddiag, float* dtable, int S, int H, int num_buckets,
                                  const RelposLut& lut, int accumulate, hipStream_t st) {
  relpos_diag_bwd_kernel<<<dim3(num_buckets, H), kWave, 0, st>>>(ddiag, dtable, S, H, num_buckets, lut,
                                                                  accumulate);
  return hipGetLastError();
}

}  // namespace t5mi
