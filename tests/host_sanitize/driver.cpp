// Host-side checker for the C ABI of include/t5mi.h, meant to be built with AddressSanitizer and
// UndefinedBehaviorSanitizer (host code only; see tests/test_host_sanitizers.py).  Every call below ends in
// the library's validation layer, before any device work, so the program runs on a host without a GPU:
// size queries, the kernel-path query, the exact-integer bucket table, and each entry point's error paths.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#include "../../include/t5mi.h"

static int failures = 0;
#define EXPECT(cond)                                                        \
  do {                                                                      \
    if (!(cond)) { std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } \
  } while (0)

static t5_block_cfg make_cfg(int B, int S, int d, int H, int dk, int F, int causal, int dtype) {
  t5_block_cfg c;
  std::memset(&c, 0, sizeof(c));
  c.batch = B; c.seq = S; c.d_model = d; c.n_heads = H; c.d_kv = dk; c.d_ff = F;
  c.num_buckets = 32; c.max_distance = 128; c.causal = causal; c.dtype = dtype;
  c.rms_eps = 1e-6f; c.attn_scale = 1.0f;
  return c;
}

int main() {
  // ---- size and path queries over a range of shapes (carving arithmetic, bucket tables)
  const int shapes[][6] = {{2, 32, 64, 4, 16, 256}, {64, 512, 512, 6, 64, 1024}, {32, 1024, 2048, 32, 64, 5120},
                           {16, 2048, 2048, 16, 128, 5120}, {1, 100, 72, 3, 24, 136}, {1, 1, 8, 1, 1, 1}};
  for (const auto& s : shapes)
    for (int causal = 0; causal < 2; ++causal)
      for (int dtype = 0; dtype < 2; ++dtype) {
        t5_block_cfg c = make_cfg(s[0], s[1], s[2], s[3], s[4], s[5], causal, dtype);
        EXPECT(t5_block_stash_bytes(&c) > 0);
        EXPECT(t5_block_workspace_bytes(&c) > 0);
        EXPECT(t5_decoder_block_stash_bytes(&c, 53) > t5_block_stash_bytes(&c));
        EXPECT(t5_decoder_block_workspace_bytes(&c, 53) > 0);
        EXPECT(t5_block_kernel_path(&c, 0) >= 0);
        EXPECT(t5_block_kernel_path(&c, 128) >= 0);
      }
  {
    t5_block_cfg xl = make_cfg(32, 1024, 2048, 32, 64, 5120, 0, T5_BF16);
    const int path = t5_block_kernel_path(&xl, 0);
    EXPECT(path == (T5_PATH_MFMA_GEMM | T5_PATH_MFMA_ATTN_FWD | T5_PATH_MFMA_ATTN_BWD));
    t5_block_cfg odd = make_cfg(1, 100, 72, 3, 24, 136, 1, T5_BF16);
    EXPECT(t5_block_kernel_path(&odd, 0) == 0);
    EXPECT(t5_block_kernel_path(nullptr, 0) == -1);
  }
  // ---- bucket tables for unusual (num_buckets, max_distance): exact integer powers inside
  const int tables[][2] = {{32, 128}, {8, 20}, {64, 1000}, {2, 3}, {256, 100000}, {32, 17}};
  for (const auto& t : tables)
    for (int bidir = 0; bidir < 2; ++bidir) {
      // n == 0: validates the table parameters and returns before touching pointers or the device
      const int rc = t5_relpos_bucket(nullptr, nullptr, 0, bidir, t[0], t[1], nullptr);
      EXPECT(rc == T5_OK || rc == T5_ERR_SHAPE || rc == T5_ERR_UNSUPPORTED);
    }
  EXPECT(t5_relpos_bucket(nullptr, nullptr, 0, 1, 31, 128, nullptr) == T5_ERR_SHAPE);   // odd and bidirectional
  EXPECT(t5_relpos_bucket(nullptr, nullptr, 0, 1, 32, 8, nullptr) == T5_ERR_SHAPE);     // max_distance too small
  EXPECT(t5_relpos_bucket(nullptr, nullptr, -1, 1, 32, 128, nullptr) == T5_ERR_SHAPE);
  EXPECT(t5_relpos_bucket(nullptr, nullptr, 5, 1, 32, 128, nullptr) == T5_ERR_NULL);

  // ---- entry points: every error path that precedes device work
  t5_block_cfg c = make_cfg(2, 32, 64, 4, 16, 256, 0, T5_F32);
  t5_block_weights w;
  t5_block_grads g;
  std::memset(&w, 0, sizeof(w));
  std::memset(&g, 0, sizeof(g));
  char dummy[64];
  EXPECT(t5_block_fwd(nullptr, dummy, &w, dummy, dummy, dummy, 1 << 20, nullptr) == T5_ERR_NULL);
  EXPECT(t5_block_fwd(&c, nullptr, &w, dummy, dummy, dummy, 1 << 20, nullptr) == T5_ERR_NULL);
  EXPECT(t5_block_fwd(&c, dummy, &w, dummy, dummy, dummy, 1 << 20, nullptr) == T5_ERR_NULL);  // weights missing
  w.ln1_scale = w.wq = w.wk = w.wv = w.wo = w.rel_table = w.ln2_scale = w.wi0 = w.wi1 = w.wo_ff = dummy;
  EXPECT(t5_block_fwd(&c, dummy, &w, dummy, dummy, dummy, 16, nullptr) == T5_ERR_WORKSPACE);
  EXPECT(t5_block_bwd(&c, dummy, dummy, &w, dummy, dummy, &g, 0, dummy, 1 << 30, nullptr) == T5_ERR_NULL);  // grads missing
  t5_block_cfg bad = c;
  bad.seq = 0;
  EXPECT(t5_block_fwd(&bad, dummy, &w, dummy, dummy, dummy, 1 << 20, nullptr) == T5_ERR_SHAPE);
  EXPECT(t5_block_stash_bytes(&bad) == 0);
  bad = c; bad.dtype = 7;
  EXPECT(t5_block_fwd(&bad, dummy, &w, dummy, dummy, dummy, 1 << 20, nullptr) == T5_ERR_UNSUPPORTED);
  bad = c; bad.dropout_rate = 1.0f;
  EXPECT(t5_block_fwd(&bad, dummy, &w, dummy, dummy, dummy, 1 << 20, nullptr) == T5_ERR_SHAPE);
  bad = c; bad.d_model = 1 << 20;
  EXPECT(t5_block_workspace_bytes(&bad) == 0);

  // ---- Adafactor
  adafactor_cfg a;
  std::memset(&a, 0, sizeof(a));
  a.lr = 1e-2f; a.decay_pow = 0.8f; a.eps1 = 1e-30f; a.eps2 = 1e-3f; a.clip = 1.0f; a.scale_by_param = 1; a.step = 1;
  float* f = reinterpret_cast<float*>(dummy);
  EXPECT(adafactor_workspace_bytes(2048, 5120, 1) > 0);
  EXPECT(adafactor_workspace_bytes(0, 5, 1) == 0);
  EXPECT(adafactor_step(f, f, f, f, nullptr, 8, 8, 1, nullptr, nullptr, dummy, 1 << 20, nullptr) == T5_ERR_NULL);
  EXPECT(adafactor_step(f, f, f, f, nullptr, 8, 8, 1, &a, nullptr, dummy, 8, nullptr) == T5_ERR_WORKSPACE);
  a.step = 0;
  EXPECT(adafactor_step(f, f, f, f, nullptr, 8, 8, 1, &a, nullptr, dummy, 1 << 20, nullptr) == T5_ERR_SHAPE);
  a.step = 1;
  EXPECT(adafactor_step(f, f, nullptr, f, nullptr, 8, 8, 1, &a, nullptr, dummy, 1 << 20, nullptr) == T5_ERR_NULL);
  EXPECT(adafactor_step_static(f, f, f, f, nullptr, 1 << 14, 1 << 14, 1, &a, nullptr, nullptr) == T5_ERR_WORKSPACE);
  EXPECT(adafactor_step_static(f, f, f, f, nullptr, 8, 8, 1, nullptr, nullptr, nullptr) == T5_ERR_NULL);
  std::vector<adafactor_tensor> ts(20);
  for (auto& t : ts) { std::memset(&t, 0, sizeof(t)); t.param = f; t.grad = f; t.v_row = f; t.v_col = f; t.rows = 64; t.cols = 300; t.factored = 1; }
  EXPECT(adafactor_multi_workspace_bytes(ts.data(), (int)ts.size()) > 0);
  EXPECT(adafactor_step_multi(ts.data(), (int)ts.size(), &a, dummy, 8, nullptr) == T5_ERR_WORKSPACE);
  ts[17].grad = nullptr;
  EXPECT(adafactor_step_multi(ts.data(), (int)ts.size(), &a, dummy, 1 << 30, nullptr) == T5_ERR_NULL);
  EXPECT(adafactor_step_multi(ts.data(), 0, &a, dummy, 1 << 30, nullptr) == T5_ERR_SHAPE);

  for (int s = 0; s < 8; ++s) EXPECT(t5_status_string(s) != nullptr && std::strlen(t5_status_string(s)) > 0);
  std::printf("%s: %d failure(s)\n", failures ? "FAILED" : "OK", failures);
  return failures ? 1 : 0;
}
