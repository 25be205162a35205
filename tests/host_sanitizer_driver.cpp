// Host-side exercise of the C ABI for an AddressSanitizer / UndefinedBehaviorSanitizer build (no GPU needed):
// argument checks, model-description checks, workspace carving arithmetic over many shapes, status strings, the
// launch-path counters, and entry points that must fail cleanly when no device is present.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>
#include "specs.h"

static int failures = 0;
#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) { std::printf("FAILED: %s (line %d)\n", #cond, __LINE__); ++failures; } \
  } while (0)

int main() {
  specs_model_desc d = {2, 64, 4, 4, 16, 256, 512, SPECS_F32, SPECS_HEAD_LM, 10000.f, 1e-6f};
  size_t prev = 0;
  for (int64_t rows : {1, 7, 64, 129, 2048, 16384, 1 << 20}) {
    size_t b = specs_workspace_bytes(&d, rows, (int32_t)(rows < 4096 ? rows : 4096));
    CHECK(b > 0 && b % 256 == 0 && b >= prev);
    prev = b;
  }
  // the benchmark shapes, both heads, both element types
  const int shapes[][7] = {{16, 1024, 16, 8, 64, 2816, 32768}, {24, 896, 14, 2, 64, 4864, 151936},
                           {28, 1536, 12, 2, 128, 8960, 151936}, {28, 3584, 28, 4, 128, 18944, 152064}};
  for (const auto& s : shapes)
    for (int dtype : {SPECS_F32, SPECS_BF16})
      for (int head : {SPECS_HEAD_LM, SPECS_HEAD_PRM}) {
        specs_model_desc m = {s[0], s[1], s[2], s[3], s[4], s[5], s[6], dtype, head, 10000.f, 1e-6f};
        size_t small = specs_workspace_bytes(&m, 256, 8), big = specs_workspace_bytes(&m, 16384, 256);
        CHECK(small > 0 && big > small);
        CHECK(specs_workspace_bytes(&m, 1LL << 31, 1 << 20) > big);          // 64-bit arithmetic, no overflow
      }
  // inconsistent descriptions and sizes
  specs_model_desc bad = d;
  bad.n_kv_heads = 3;
  CHECK(specs_workspace_bytes(&bad, 64, 1) == 0);
  bad = d; bad.head_dim = 15;
  CHECK(specs_workspace_bytes(&bad, 64, 1) == 0);
  bad = d; bad.ffn = 100;
  CHECK(specs_workspace_bytes(&bad, 64, 1) == 0);
  bad = d; bad.dtype = 7;
  CHECK(specs_workspace_bytes(&bad, 64, 1) == 0);
  bad = d; bad.rope_base = -1.f;
  CHECK(specs_workspace_bytes(&bad, 64, 1) == 0);
  CHECK(specs_workspace_bytes(&d, 0, 1) == 0 && specs_workspace_bytes(&d, 64, 0) == 0 && specs_workspace_bytes(nullptr, 64, 1) == 0);
  // null / invalid arguments never reach a device
  specs_ctx* ctx = nullptr;
  CHECK(specs_ctx_create(0, nullptr, nullptr, 0, &ctx) == SPECS_EINVAL);
  alignas(256) static char fake_ws[512];
  CHECK(specs_ctx_create(0, nullptr, fake_ws + 1, 256, &ctx) == SPECS_EINVAL);    // misaligned workspace
  int rc = specs_ctx_create(0, nullptr, fake_ws, sizeof(fake_ws), &ctx);          // no GPU here: a clean HIP error
  CHECK(rc == SPECS_EHIP || rc == SPECS_OK);
  if (rc == SPECS_OK) CHECK(specs_ctx_destroy(ctx) == SPECS_OK);
  CHECK(specs_ctx_destroy(nullptr) == SPECS_OK);
  CHECK(specs_model_destroy(nullptr) == SPECS_OK && specs_prefix_destroy(nullptr) == SPECS_OK);
  CHECK(specs_score_blocks(nullptr, nullptr, nullptr, nullptr, 1, 1, nullptr, nullptr) == SPECS_EINVAL);
  CHECK(specs_score_blocks_static(nullptr, nullptr, nullptr, nullptr, 1, 1, nullptr, nullptr) == SPECS_EINVAL);
  CHECK(specs_op_qkv_rope(nullptr, nullptr, nullptr, nullptr, nullptr, 1, 1, nullptr, nullptr, nullptr) == SPECS_EINVAL);
  CHECK(specs_score_target_and_reward(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 1, 1, nullptr, nullptr,
                                      nullptr) == SPECS_EINVAL);
  CHECK(specs_generate_blocks(nullptr, nullptr, nullptr, 1, 1, 0, nullptr, nullptr, nullptr, nullptr) == SPECS_EINVAL);
  CHECK(specs_commit_block(nullptr, nullptr, nullptr, nullptr) == SPECS_EINVAL);
  CHECK(specs_commit_block_dev(nullptr, nullptr, nullptr, nullptr) == SPECS_EINVAL);
  CHECK(specs_subsample(nullptr, nullptr, nullptr, nullptr, nullptr, 1, 1, nullptr, 1, nullptr, nullptr, nullptr) == SPECS_EINVAL);
  CHECK(specs_select_and_switch(nullptr, nullptr, nullptr, nullptr, nullptr, 1, 1, 1.f, 0.5f, nullptr, nullptr, nullptr,
                                nullptr) == SPECS_EINVAL);
  CHECK(specs_prefill(nullptr, nullptr, nullptr, nullptr) == SPECS_EINVAL);
  CHECK(specs_op_linear(nullptr, SPECS_BF16, nullptr, nullptr, 1, 1, 1, nullptr, 0) == SPECS_EINVAL);
  CHECK(specs_ctx_status(nullptr, nullptr) == SPECS_EINVAL && specs_ctx_profile(nullptr, 1) == SPECS_EINVAL);
  // status strings and path counters
  for (int c = -3; c < 40; ++c) CHECK(specs_strerror(c) != nullptr && std::strlen(specs_strerror(c)) > 0);
  int32_t counts[SPECS_PATH_COUNT];
  CHECK(specs_path_counts(counts, 1) == SPECS_OK && specs_path_counts(nullptr, 0) == SPECS_EINVAL);
  CHECK(specs_path_counts(counts, 0) == SPECS_OK);
  for (int i = 0; i < SPECS_PATH_COUNT; ++i) CHECK(counts[i] == 0);
  std::printf(failures ? "host ABI driver: %d failure(s)\n" : "host ABI driver: ok\n", failures);
  return failures ? 1 : 0;
}
