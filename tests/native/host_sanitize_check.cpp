// Drives the C ABI through a randomised sequence of plans, decode steps and inspections.  It is linked against a build
// of the library's host code with AddressSanitizer and UndefinedBehaviorSanitizer (host side only), so any host-memory
// error or undefined arithmetic in the bookkeeping aborts the run.  Results are not checked here (the parity tests do
// that); statuses are.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include <unistd.h>

#include "../../include/tkv.h"

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) { std::printf("FAILED %s (line %d)\n", #cond, __LINE__); std::exit(1); } \
  } while (0)
#define OK(call)                                                                                              \
  do {                                                                                                        \
    tkv_status s_ = (call);                                                                                   \
    if (s_ != TKV_OK) { std::printf("%s -> %d: %s (line %d)\n", #call, s_, tkv_last_error(c), __LINE__); std::exit(1); } \
  } while (0)

static uint16_t bf16_of(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

static void run_mode(int mode) {
  const int L = 3, B = 2, Hq = 8, Hkv = 2, D = 64, N0 = 400, NMAX = 460;
  tkv_config cfg;
  std::memset(&cfg, 0, sizeof cfg);
  cfg.n_layers = L; cfg.batch = B; cfg.n_q_heads = Hq; cfg.n_kv_heads = Hkv; cfg.head_dim = D; cfg.max_tokens = NMAX;
  cfg.kv_dtype = TKV_BF16; cfg.out_dtype = TKV_F32; cfg.t2_format = mode == 1 ? TKV_T2_INT4_G32 : TKV_T2_INT8_ROW;
  cfg.k_sink = 4; cfg.k_window = 16; cfg.prefetch_mode = mode;
  cfg.scorer = mode == 1 ? TKV_SCORE_VATP : mode == 2 ? TKV_SCORE_COMBINED : TKV_SCORE_REDUNDANCY;
  cfg.redundancy_weight = mode == 0 ? 0.f : 1.5f;       // 0: the default weight
  cfg.host_rows = 480;                       // small: the store is rewritten every few plans
  tkv_cache* c = nullptr;
  CHECK(tkv_create(&cfg, &c) == TKV_OK && c);
  std::mt19937 rng(7 + mode);
  std::normal_distribution<float> nd(0.f, 1.f);
  auto fill = [&](std::vector<uint16_t>& h) { for (auto& x : h) x = bf16_of(nd(rng)); };
  uint16_t *dk, *dv, *dq; float* dout;
  const size_t ctx = (size_t)B * N0 * Hkv * D, step = (size_t)L * B * Hkv * D, qn = (size_t)L * B * Hq * D;
  CHECK(hipMalloc(&dk, ctx * 2) == hipSuccess && hipMalloc(&dv, ctx * 2) == hipSuccess);
  CHECK(hipMalloc(&dq, qn * 2) == hipSuccess && hipMalloc(&dout, qn * 4) == hipSuccess);
  std::vector<uint16_t> h(ctx);
  for (int l = 0; l < L; ++l) {
    fill(h);
    CHECK(hipMemcpy(dk, h.data(), ctx * 2, hipMemcpyHostToDevice) == hipSuccess);
    fill(h);
    CHECK(hipMemcpy(dv, h.data(), ctx * 2, hipMemcpyHostToDevice) == hipSuccess);
    OK(tkv_append(c, l, dk, dv, N0, nullptr));
  }
  int n = N0;
  std::vector<uint8_t> tiers((size_t)B * NMAX, 0), got((size_t)B * NMAX);
  std::vector<float> scores((size_t)B * NMAX);
  std::vector<int32_t> list(NMAX);
  std::vector<uint16_t> hs(step), hq(qn);
  std::vector<char> row(D * 2), codes(D), scales(16);
  for (int round = 0; round < 14; ++round) {
    for (int b = 0; b < B; ++b)
      for (int i = 4; i < n - 16; ++i) {
        uint8_t& t = tiers[(size_t)b * NMAX + i];
        if (t == 3 || rng() % 100 >= 40) continue;
        const unsigned r = rng() % 100;
        t = r < 30 ? 0 : r < 65 ? 1 : r < 92 ? 2 : 3;
      }
    OK(tkv_set_tiers(c, tiers.data()));
    OK(tkv_migrate(c, nullptr));
    if (round % 3 == 0) OK(tkv_wait_prefetch(c));
    fill(hs);
    CHECK(hipMemcpy(dk, hs.data(), step * 2, hipMemcpyHostToDevice) == hipSuccess);
    fill(hs);
    CHECK(hipMemcpy(dv, hs.data(), step * 2, hipMemcpyHostToDevice) == hipSuccess);
    fill(hq);
    CHECK(hipMemcpy(dq, hq.data(), qn * 2, hipMemcpyHostToDevice) == hipSuccess);
    if (round % 2) {
      OK(tkv_decode_step(c, dk, dv, dq, dout, nullptr));
    } else {
      for (int l = 0; l < L; ++l) {
        OK(tkv_append(c, l, dk + (size_t)l * B * Hkv * D, dv + (size_t)l * B * Hkv * D, 1, nullptr));
        OK(tkv_attend_and_score(c, l, dq + (size_t)l * B * Hq * D, dout + (size_t)l * B * Hq * D, nullptr));
      }
    }
    ++n;
    OK(tkv_get_tiers(c, got.data()));
    for (int b = 0; b < B; ++b) CHECK(std::memcmp(&got[(size_t)b * NMAX], &tiers[(size_t)b * NMAX], n - 1) == 0);
    OK(tkv_get_scores(c, scores.data()));
    int32_t cnt = 0, total = 0;
    for (int t = 0; t < 4; ++t) { OK(tkv_get_index_list(c, t, 1, list.data(), &cnt)); total += cnt; }
    CHECK(total == n);
    for (int i = 4; i < n - 16; i += 37) {
      const uint8_t t = tiers[(size_t)1 * NMAX + i];
      if (t <= 1) OK(tkv_get_row(c, 2, 1, 1, i, 1, row.data()));
      if (t == 2) OK(tkv_get_t2_row(c, 2, 1, 1, i, 0, codes.data(), scales.data()));
    }
    tkv_stats st;
    OK(tkv_get_stats(c, &st));
    CHECK(st.tier_count[0] + st.tier_count[1] + st.tier_count[2] + st.tier_count[3] == (int64_t)B * n);
    tkv_policy pol = {300000, 400000, 250000, 50000, (uint32_t)(round & 1)};
    if (round == 13) { OK(tkv_classify(c, &pol, nullptr)); OK(tkv_migrate(c, nullptr)); }
  }
  tkv_stats st;
  OK(tkv_get_stats(c, &st));
  std::printf("mode %d: %lld migrates, store rewritten %lld times, %lld rows of it in use, h2d %lld B, d2h %lld B\n", mode,
              (long long)st.n_migrate, (long long)st.n_rehome, (long long)st.host_rows_used, (long long)st.h2d_bytes,
              (long long)st.d2h_bytes);
  CHECK(st.n_rehome + st.n_repack >= 1);
  // two query tokens per sequence at once, over two positions appended after the last migrate
  for (int l = 0; l < L; ++l) OK(tkv_append(c, l, dk, dv, 2, nullptr));
  for (int l = 0; l < L; ++l) OK(tkv_attend_and_score_chunk(c, l, dq, dout, 2, nullptr));
  CHECK(tkv_attend_and_score_chunk(c, 0, dq, dout, 3, nullptr) == TKV_ESTATE);
  CHECK(tkv_attend_and_score_chunk(c, 0, dq, dout, 0, nullptr) == TKV_EINVAL);
  OK(tkv_get_scores(c, scores.data()));
  // error paths on a live handle
  CHECK(tkv_attend_and_score(c, 99, dq, dout, nullptr) == TKV_EINVAL);
  CHECK(tkv_migrate(c, nullptr) == TKV_ESTATE);
  tkv_policy bad = {1, 2, 3, 4, 0};
  CHECK(tkv_classify(c, &bad, nullptr) == TKV_EINVAL);
  CHECK(tkv_append(c, 0, dk, dv, NMAX, nullptr) == TKV_ECAPACITY);
  tkv_destroy(c);
  (void)hipFree(dk); (void)hipFree(dv); (void)hipFree(dq); (void)hipFree(dout);
}

int main(int argc, char** argv) {
  const bool host_only = argc > 1 && std::strcmp(argv[1], "--host-only") == 0;
  // host-only validation first (no handle)
  tkv_cache* c = nullptr;
  tkv_config bad;
  std::memset(&bad, 0, sizeof bad);
  CHECK(tkv_create(&bad, &c) == TKV_EINVAL && c == nullptr);
  CHECK(tkv_create(nullptr, &c) == TKV_EINVAL);
  int64_t out[4];
  tkv_policy pol = {300000, 520000, 150000, 30000, 1};
  CHECK(tkv_tier_counts(&pol, 4000, 100, out) == TKV_OK && out[0] + out[1] + out[2] + out[3] == 4000);
  tkv_destroy(nullptr);
  tkv_config cfg;
  std::memset(&cfg, 0, sizeof cfg);
  cfg.n_layers = 1; cfg.batch = 1; cfg.n_q_heads = 9; cfg.n_kv_heads = 2; cfg.head_dim = 64; cfg.max_tokens = 64;
  CHECK(tkv_create(&cfg, &c) == TKV_EINVAL && c == nullptr);      // heads not a multiple of kv heads
  cfg.n_q_heads = 8; cfg.head_dim = 96;
  CHECK(tkv_create(&cfg, &c) == TKV_EINVAL && c == nullptr);      // unsupported head_dim
  cfg.head_dim = 64; cfg.prefetch_mode = 7;
  CHECK(tkv_create(&cfg, &c) == TKV_EINVAL && c == nullptr);
  CHECK(tkv_last_error(nullptr) != nullptr);
  for (int mode = 0; mode < 3 && !host_only; ++mode) run_mode(mode);
  std::printf("host sanitizer check passed\n");
  std::fflush(stdout);
  // leave without running the HIP runtime's own exit handlers: their frees trip the sanitizer's allocator checks now
  // and then, and they are not what is under test
  _exit(0);
}
