// Host-only walk through the argument checks of the C ABI, built with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host code (tests/test_abi_host.py builds and runs it; no GPU is needed:
// every call here is rejected, or answered, before anything touches a device).
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <limits>

#include "../../include/ddd.h"
#include "../../include/ddd_body.h"

static int failures = 0;
#define CHECK(cond)                                                    \
  do {                                                                 \
    if (!(cond)) {                                                     \
      std::printf("FAILED line %d: %s\n", __LINE__, #cond);            \
      ++failures;                                                      \
    }                                                                  \
  } while (0)

int main() {
  ddd_config ok = {1, 4096, 32000, 10, 10, 60, 0.3f, 0xFFFFFFFFu, 0u};
  CHECK(ddd_config_validate(&ok) == DDD_OK);
  CHECK(ddd_pool_capacity(&ok) == 911);
  CHECK(ddd_scratch_bytes(&ok) > 0);
  CHECK(ddd_config_validate(nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_pool_capacity(nullptr) == 0 && ddd_scratch_bytes(nullptr) == 0);

  // every field pushed over its limits, including values whose products overflow 32 bits
  const int32_t extremes[] = {std::numeric_limits<int32_t>::min(), -1, 0, std::numeric_limits<int32_t>::max()};
  for (int field = 0; field < 6; ++field)
    for (int32_t x : extremes) {
      ddd_config c = ok;
      (&c.B)[field] = x;
      CHECK(ddd_config_validate(&c) == DDD_ERR_INVALID_ARG);
      CHECK(ddd_pool_capacity(&c) == 0 && ddd_scratch_bytes(&c) == 0);
    }
  {
    ddd_config c = ok;   // the largest pool and batch the limits allow: sizes are computed without overflow
    c.B = DDD_BMAX; c.k = DDD_KWIDE_MAX; c.H = 4096; c.V = 1000; c.max_depth = 4; c.m = DDD_MMAX;
    CHECK(ddd_config_validate(&c) == DDD_ERR_INVALID_ARG);     // hidden rows beyond 32-bit byte offsets
    c.B = DDD_BMAX - 1;
    CHECK(ddd_config_validate(&c) == DDD_OK);
    CHECK(ddd_pool_capacity(&c) == 1u + 128u + 3u * 128u * 128u);
    CHECK(ddd_scratch_bytes(&c) > (size_t)c.B * c.k * c.V * sizeof(float));
    c.threshold = std::nanf("");
    CHECK(ddd_config_validate(&c) == DDD_ERR_INVALID_ARG);
    c.threshold = 0.5f; c.flags = 4u;
    CHECK(ddd_config_validate(&c) == DDD_ERR_INVALID_ARG);
  }
  for (int code = 1; code >= -9; --code) CHECK(std::strlen(ddd_strerror(code)) > 0);
  CHECK(ddd_last_hip_error() != nullptr);

  // null and out-of-range arguments: every entry point answers with a status and touches nothing
  ddd_ctx* ctx = nullptr;
  CHECK(ddd_create(nullptr, &ctx) == DDD_ERR_INVALID_ARG && ctx == nullptr);
  CHECK(ddd_create(&ok, nullptr) == DDD_ERR_INVALID_ARG);
  const int rc = ddd_create(&ok, &ctx);          // no device here: a status, not a crash (a GPU machine may create it)
  CHECK(rc == DDD_ERR_NO_DEVICE || rc == DDD_ERR_WRONG_ARCH || rc == DDD_ERR_HIP || rc == DDD_OK);
  if (rc == DDD_OK) CHECK(ddd_destroy(ctx) == DDD_OK);
  CHECK(ddd_destroy(nullptr) == DDD_ERR_INVALID_ARG);
  ddd_state st;
  ddd_tree tr;
  std::memset(&st, 0, sizeof(st));
  std::memset(&tr, 0, sizeof(tr));
  int32_t word = 0;
  float f = 0.f;
  CHECK(ddd_round_reset(nullptr, &st, nullptr, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_lmhead_topk(nullptr, &word, &word, 1, nullptr, &word, &f, &f, nullptr, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_beam_select(nullptr, 0, &word, &f, &st, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_depth_continue(nullptr, 1, &st, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_draft_step(nullptr, 0, &word, &word, &st, &tr, nullptr, nullptr, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_tree_finalize(nullptr, &st, &tr, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_verify_accept(nullptr, &tr, &word, &word, &word, &word, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_verify_sample(nullptr, &tr, &f, 1.0f, nullptr, nullptr, &word, &word, &word, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_round_enqueue(nullptr, &word, &st, &tr, nullptr, &word, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                          nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_round_run(nullptr, &word, &st, &tr, nullptr, &word, nullptr, nullptr, nullptr, nullptr, nullptr) ==
        DDD_ERR_INVALID_ARG);
  CHECK(ddd_round_capture(nullptr, &word, &st, &tr, nullptr, &word, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                          &word) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_round_launch(nullptr, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_round_run_stats(nullptr, nullptr, nullptr, nullptr, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_weights_pack(nullptr, &word, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_num_slices(nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_tree_attention_workspace(nullptr, 32, 256) == 0);
  CHECK(ddd_kv_pack(nullptr, &word, &word, 1, 1, &word, &word, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_tree_attention(nullptr, &tr, &word, &word, &word, &word, &word, 1, 1, &word, 16, &f, nullptr) ==
        DDD_ERR_INVALID_ARG);
  CHECK(ddd_profile_lmhead(nullptr, &word, &word, 1, 1, &f, &f, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_trace_enable(nullptr, 1) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_stats_bind(nullptr, nullptr) == DDD_ERR_INVALID_ARG);
  uint64_t w64 = 0;
  CHECK(ddd_trace_read(nullptr, &w64, 1) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_trace_words() == (size_t)(DDD_DMAX + 1) * DDD_TRACE_CALL_WORDS);
  // the allocation-free entry point: limits and nulls are answered before a device is looked for
  CHECK(ddd_static_scratch_bytes() == (size_t)16 * 16 * 256 * 8 + 16 * 256 * 4);
  ddd_config tiny = {1, 256, 1000, 4, 6, 16, 0.35f, 0xFFFFFFFFu, 0u};
  CHECK(ddd_lmhead_topk_static(nullptr, &word, &word, 1, nullptr, &word, &f, &f, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_lmhead_topk_static(&tiny, nullptr, &word, 1, nullptr, &word, &f, &f, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_lmhead_topk_static(&tiny, &word, &word, 0, nullptr, &word, &f, &f, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_lmhead_topk_static(&tiny, &word, &word, DDD_STATIC_ROWS + 1, nullptr, &word, &f, &f, nullptr) ==
        DDD_ERR_STATIC_LIMIT);
  tiny.k = DDD_KMAX + 1;
  CHECK(ddd_lmhead_topk_static(&tiny, &word, &word, 1, nullptr, &word, &f, &f, nullptr) == DDD_ERR_STATIC_LIMIT);
  // the draft layer's host side
  ddd_body* body = nullptr;
  ddd_body_config bad = {0, 4, 256, 256, 10, 2, 0};
  CHECK(ddd_body_create(nullptr, &body) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_body_create(&bad, &body) == DDD_ERR_INVALID_ARG && body == nullptr);
  bad.B = 4097; bad.k = 2;
  CHECK(ddd_body_create(&bad, &body) == DDD_ERR_INVALID_ARG);
  bad.B = std::numeric_limits<int32_t>::max(); bad.k = std::numeric_limits<int32_t>::max();
  CHECK(ddd_body_create(&bad, &body) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_body_destroy(nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_body_bind(nullptr, nullptr, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_body_step(nullptr, 0, &st, &word, nullptr) == DDD_ERR_INVALID_ARG);
  CHECK(ddd_body_linear(nullptr, &word, 16, 128, &word, 1, &f, 0, nullptr) == DDD_ERR_INVALID_ARG);

  std::printf(failures == 0 ? "ABI_SANITIZE_OK\n" : "ABI_SANITIZE_FAILED (%d)\n", failures);
  return failures == 0 ? 0 : 1;
}
