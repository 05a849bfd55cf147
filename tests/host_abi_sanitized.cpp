// Host-side exercise of the C ABI for a build with the address and undefined-behaviour sanitizers
// on the host code (tests/test_host_sanitized.py compiles and runs it).  It walks the paths that run
// without a GPU: configuration checks, plan creation for all workload shapes (tables, block budget,
// work tables), info, permutation export, error texts, NULL arguments, destroy.  On a machine with
// a GPU the same calls also cover the table uploads.  Prints one line per group; exit code 0 = all
// expectations held (the sanitizers abort with their own report otherwise).
#include <cmath>
#include <cstdio>
#include <cstring>
#include <vector>

#include "rf2.h"

static int failures = 0;
#define EXPECT(cond)                                                        \
  do {                                                                      \
    if (!(cond)) { std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } \
  } while (0)

static rf2_config base_config() {
  rf2_config c;
  std::memset(&c, 0, sizeof c);
  c.batch = 1; c.heads = 2; c.head_dim = 64; c.T = 6; c.H = 16; c.W = 16; c.block = 64;
  c.sink_frames = 1; c.sink_at_end = 1; c.sparsity = 0.5f;
  return c;
}

static void check_plan(const rf2_config& c) {
  rf2_plan* p = nullptr;
  const int rc = rf2_plan_create(&c, &p);
  EXPECT(rc == RF2_OK && p != nullptr);
  if (rc != RF2_OK) return;
  rf2_info in;
  EXPECT(rf2_plan_info(p, &in) == RF2_OK);
  const long long N = (long long)c.T * c.H * c.W + c.text_tokens;
  EXPECT(in.N == N && in.N_pad >= N && in.N_pad - N < c.block);
  EXPECT(in.n_blocks == (N + c.block - 1) / c.block);
  EXPECT(in.k_row >= 1 && in.k_row <= in.n_blocks_k);
  std::vector<int32_t> perm((size_t)N), inv((size_t)N);
  EXPECT(rf2_plan_perm(p, perm.data(), inv.data()) == RF2_OK);
  std::vector<char> seen((size_t)N, 0);
  bool bijection = true;
  for (long long i = 0; i < N; ++i) {
    const int32_t n = perm[(size_t)i];
    if (n < 0 || n >= N || seen[(size_t)n] || inv[(size_t)n] != i) { bijection = false; break; }
    seen[(size_t)n] = 1;
  }
  EXPECT(bijection);
  EXPECT(rf2_plan_perm(p, nullptr, nullptr) == RF2_OK);          // both outputs optional
  // compute calls on a plan: NULL tensors are rejected before anything else happens
  EXPECT(rf2_permute(p, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == RF2_ERR_INVALID_ARG);
  EXPECT(rf2_predict_mask(p, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == RF2_ERR_INVALID_ARG);
  EXPECT(rf2_block_sparse_attn(p, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == RF2_ERR_INVALID_ARG);
  EXPECT(rf2_block_sparse_attn_unpermuted(p, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == RF2_ERR_INVALID_ARG);
  EXPECT(rf2_unpermute(p, nullptr, nullptr, nullptr) == RF2_ERR_INVALID_ARG);
  EXPECT(rf2_plan_destroy(p) == RF2_OK);
}

int main() {
  // 1. the workload shapes (tiny, image, 480p, 720p, long video) and the variants of the configuration
  struct Shape { int heads, d, T, H, W, block, sink; float s; };
  const Shape shapes[] = {{2, 64, 6, 16, 16, 64, 1, 0.5f},   {24, 128, 1, 64, 64, 128, 0, 0.5f},
                          {40, 128, 21, 30, 52, 128, 1, 0.8f}, {40, 128, 21, 45, 80, 128, 1, 0.8f},
                          {24, 128, 33, 45, 80, 128, 1, 0.9f}, {3, 128, 5, 10, 13, 128, 1, 0.5f},
                          {1, 128, 1, 5, 7, 128, 0, 0.5f},     {2, 64, 7, 10, 13, 64, 2, 0.3f}};
  for (const Shape& sh : shapes) {
    rf2_config c = base_config();
    c.heads = sh.heads; c.head_dim = sh.d; c.T = sh.T; c.H = sh.H; c.W = sh.W; c.block = sh.block;
    c.sink_frames = sh.sink; c.sparsity = sh.s;
    check_plan(c);
    c.qkv_layout = RF2_LAYOUT_BNHD; c.text_tokens = 77;
    check_plan(c);
    c.select_mode = RF2_SELECT_CDF; c.cdf_threshold = 0.9f;
    check_plan(c);
    c.select_mode = RF2_SELECT_TOPN; c.text_tokens = 0; c.block_k = sh.block == 64 ? 128 : 64;
    check_plan(c);
    c.block = 256; c.block_k = 128; c.budget_mode = RF2_BUDGET_ROW_PLUS_SINK;
    check_plan(c);
    if (sh.sink) { c = base_config(); c.T = sh.T; c.H = sh.H; c.W = sh.W; c.sink_frames = sh.sink; c.sink_at_end = 0; c.wt = 2; c.wh = 3; c.ww = 5; check_plan(c); }
  }
  std::printf("plans: %s\n", failures ? "FAILED" : "ok");

  // 2. configurations that must be refused, with the code the header promises
  rf2_plan* p = nullptr;
  rf2_config c = base_config();
  EXPECT(rf2_plan_create(nullptr, &p) == RF2_ERR_INVALID_ARG);
  EXPECT(rf2_plan_create(&c, nullptr) == RF2_ERR_INVALID_ARG);
  c = base_config(); c.batch = 0;            EXPECT(rf2_plan_create(&c, &p) == RF2_ERR_INVALID_ARG && p == nullptr);
  c = base_config(); c.sink_frames = 6;      EXPECT(rf2_plan_create(&c, &p) == RF2_ERR_INVALID_ARG);
  c = base_config(); c.sparsity = 1.0f;      EXPECT(rf2_plan_create(&c, &p) == RF2_ERR_INVALID_ARG);
  c = base_config(); c.sparsity = NAN;       EXPECT(rf2_plan_create(&c, &p) == RF2_ERR_INVALID_ARG);
  c = base_config(); c.wt = -1;              EXPECT(rf2_plan_create(&c, &p) == RF2_ERR_INVALID_ARG);
  c = base_config(); c.wt = 2;               EXPECT(rf2_plan_create(&c, &p) == RF2_ERR_INVALID_ARG);   // wh, ww left 0
  c = base_config(); c.budget_mode = 7;      EXPECT(rf2_plan_create(&c, &p) == RF2_ERR_INVALID_ARG);
  c = base_config(); c.select_mode = RF2_SELECT_CDF; c.cdf_threshold = 1.0f; EXPECT(rf2_plan_create(&c, &p) == RF2_ERR_INVALID_ARG);
  c = base_config(); c.head_dim = 96;        EXPECT(rf2_plan_create(&c, &p) == RF2_ERR_UNSUPPORTED);
  c = base_config(); c.block = 32;           EXPECT(rf2_plan_create(&c, &p) == RF2_ERR_UNSUPPORTED);
  c = base_config(); c.block = 256;          EXPECT(rf2_plan_create(&c, &p) == RF2_ERR_UNSUPPORTED);
  c = base_config(); c.T = 4096; c.H = 256; c.W = 256; EXPECT(rf2_plan_create(&c, &p) == RF2_ERR_UNSUPPORTED);
  c = base_config(); c.text_tokens = 5; c.sink_at_end = 0; EXPECT(rf2_plan_create(&c, &p) == RF2_ERR_UNSUPPORTED);
  c = base_config(); c.heads = 70000;        EXPECT(rf2_plan_create(&c, &p) == RF2_ERR_UNSUPPORTED);
  std::printf("refusals: %s\n", failures ? "FAILED" : "ok");

  // 3. NULL plans and error texts
  rf2_info in;
  EXPECT(rf2_plan_info(nullptr, &in) == RF2_ERR_INVALID_ARG);
  EXPECT(rf2_plan_perm(nullptr, nullptr, nullptr) == RF2_ERR_INVALID_ARG);
  EXPECT(rf2_plan_destroy(nullptr) == RF2_OK);
  EXPECT(rf2_unpermute(nullptr, nullptr, nullptr, nullptr) == RF2_ERR_INVALID_ARG);
  EXPECT(rf2_measure_peaks(nullptr, nullptr, nullptr) == RF2_ERR_INVALID_ARG);
  for (int code = 1; code >= -6; --code) EXPECT(rf2_strerror(code) != nullptr && std::strlen(rf2_strerror(code)) > 0);
  EXPECT(rf2_version() >= 100);
  std::printf("null and error paths: %s\n", failures ? "FAILED" : "ok");
  std::printf(failures ? "HOST ABI CHECK FAILED (%d)\n" : "HOST ABI CHECK PASSED\n", failures);
  return failures ? 1 : 0;
}
