// Host-side checks of libcamera_hip's C ABI, meant to run under AddressSanitizer / UndefinedBehaviorSanitizer on a
// machine without a GPU: every call below is refused (or is a no-op) by the argument validation that runs before any
// GPU work, so only host code executes.  Pointers marked FAKE are never dereferenced by the library.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/camera.h"

static int failures = 0;
#define EXPECT(cond)                                                       \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      ++failures;                                                          \
    }                                                                      \
  } while (0)

int main() {
  void* const FAKE = reinterpret_cast<void*>(0x1000);
  camera_ctx* ctx = nullptr;
  EXPECT(camera_create(nullptr, 0) == CAMERA_EINVAL);
  EXPECT(camera_create(&ctx, -1) == CAMERA_EINVAL && std::strstr(camera_last_error(nullptr), "device"));
  EXPECT(camera_create(&ctx, 0) == CAMERA_OK && ctx != nullptr);
  EXPECT(camera_version() == 1);

  // routing
  EXPECT(camera_route_topk(ctx, nullptr, FAKE, 7, 16, 64, 64, FAKE, 64, nullptr, 8, 2, 1, (int32_t*)FAKE, (float*)FAKE) == CAMERA_EDTYPE);
  EXPECT(camera_route_topk(ctx, nullptr, FAKE, CAMERA_BF16, 16, 60, 64, FAKE, 64, nullptr, 8, 2, 1, (int32_t*)FAKE, (float*)FAKE) == CAMERA_ESHAPE);
  EXPECT(camera_route_topk(ctx, nullptr, FAKE, CAMERA_BF16, 16, 64, 64, FAKE, 64, nullptr, 300, 2, 1, (int32_t*)FAKE, (float*)FAKE) == CAMERA_EUNSUPPORTED);
  EXPECT(camera_route_topk(ctx, nullptr, FAKE, CAMERA_BF16, 0, 64, 64, FAKE, 64, nullptr, 8, 2, 1, (int32_t*)FAKE, (float*)FAKE) == CAMERA_OK);
  EXPECT(std::strlen(camera_last_error(ctx)) < 512);

  // scoring: every refusal path of the shape / pointer checks
  auto score = [&](int64_t n, int64_t d, int64_t f, int ne, int k, float alpha, int flags, int64_t sgu) {
    return camera_score_layer(ctx, nullptr, FAKE, CAMERA_BF16, n, d, d, (int32_t*)FAKE, (float*)FAKE, k, ne, f, FAKE, FAKE, sgu, FAKE,
                              f * d, alpha, flags, (float*)FAKE, (float*)FAKE, (float*)FAKE, (float*)FAKE);
  };
  EXPECT(score(16, 64, 32, 8, 2, 1.5f, 0, 32 * 64) == CAMERA_EINVAL);
  EXPECT(score(16, 64, 32, 8, 9, 0.5f, 0, 32 * 64) == CAMERA_EINVAL);
  EXPECT(score(16, 64, 32, 8, 2, 0.5f, 64, 32 * 64) == CAMERA_EINVAL);
  EXPECT(score(16, 64, 32, 8, 2, 0.5f, 0, 32 * 64 - 8) == CAMERA_ESHAPE);
  EXPECT(score(int64_t(1) << 31, 64, 32, 8, 2, 0.5f, 0, 32 * 64) == CAMERA_ESHAPE);
  EXPECT(score(int64_t(1) << 24, 64, 32, 8, 8, 0.5f, 0, 32 * 64) == CAMERA_EUNSUPPORTED);

  // ranking: segment tables at their limits, ratios, levels
  std::vector<int64_t> seg(CAMERA_MAX_SEGMENTS + 2);
  for (size_t i = 0; i < seg.size(); ++i) seg[i] = (int64_t)i * 3;
  const int64_t n_full = seg[CAMERA_MAX_SEGMENTS];
  EXPECT(camera_select_prune(ctx, nullptr, (float*)FAKE, n_full, seg.data(), CAMERA_MAX_SEGMENTS + 1, 0.4, (uint8_t*)FAKE,
                             (int32_t*)FAKE, nullptr, nullptr) == CAMERA_EUNSUPPORTED);
  EXPECT(camera_select_prune(ctx, nullptr, (float*)FAKE, n_full + 1, seg.data(), CAMERA_MAX_SEGMENTS, 0.4, (uint8_t*)FAKE,
                             (int32_t*)FAKE, nullptr, nullptr) == CAMERA_EINVAL);
  EXPECT(camera_select_prune(ctx, nullptr, (float*)FAKE, n_full, seg.data(), CAMERA_MAX_SEGMENTS, 1.0001, (uint8_t*)FAKE,
                             (int32_t*)FAKE, nullptr, nullptr) == CAMERA_EINVAL);
  seg[5] = 1;  // falls
  EXPECT(camera_select_prune(ctx, nullptr, (float*)FAKE, n_full, seg.data(), CAMERA_MAX_SEGMENTS, 0.4, (uint8_t*)FAKE,
                             (int32_t*)FAKE, nullptr, nullptr) == CAMERA_EINVAL);
  const int64_t seg2[3] = {0, 40, 100};
  const double ratios7[7] = {0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7};
  const double ratios8[8] = {0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8};
  EXPECT(camera_select_prune_multi(ctx, nullptr, (float*)FAKE, 100, seg2, 2, 8, ratios8, (uint8_t*)FAKE, (int32_t*)FAKE) == CAMERA_EUNSUPPORTED);
  EXPECT(camera_select_prune_multi(ctx, nullptr, nullptr, 100, seg2, 2, 7, ratios7, (uint8_t*)FAKE, (int32_t*)FAKE) == CAMERA_EINVAL);
  const int bits8[8] = {8, 7, 6, 5, 4, 3, 2, 1};
  const double lev8[8] = {0.125, 0.125, 0.125, 0.125, 0.125, 0.125, 0.125, 0.125};
  EXPECT(camera_alloc_bits(ctx, nullptr, nullptr, 100, seg2, 2, 8, bits8, lev8, (uint8_t*)FAKE, (int32_t*)FAKE, nullptr) == CAMERA_EINVAL);
  EXPECT(camera_alloc_bits(ctx, nullptr, (float*)FAKE, 100, seg2, 2, 9, bits8, lev8, (uint8_t*)FAKE, (int32_t*)FAKE, nullptr) == CAMERA_EUNSUPPORTED);
  const double lev_bad[3] = {0.5, 0.3, 0.3};
  EXPECT(camera_alloc_bits(ctx, nullptr, (float*)FAKE, 100, seg2, 2, 3, bits8, lev_bad, (uint8_t*)FAKE, (int32_t*)FAKE, nullptr) == CAMERA_EINVAL);
  EXPECT(camera_rank_decisions(ctx, nullptr, (float*)FAKE, 100, seg2, 2, 7, ratios7, (uint8_t*)FAKE, (int32_t*)FAKE, 3, bits8, lev_bad,
                               (uint8_t*)FAKE, (int32_t*)FAKE, nullptr) == CAMERA_EUNSUPPORTED);
  EXPECT(camera_rank_decisions(ctx, nullptr, nullptr, 100, seg2, 2, 2, ratios7, (uint8_t*)FAKE, (int32_t*)FAKE, 3, bits8, lev8,
                               (uint8_t*)FAKE, (int32_t*)FAKE, nullptr) == CAMERA_EINVAL);
  EXPECT(camera_select_prune_noalloc(ctx, nullptr, (float*)FAKE, (int64_t(1) << 20) + 1, seg2, 2, 0.4, (uint8_t*)FAKE, (int32_t*)FAKE,
                                     nullptr) == CAMERA_EUNSUPPORTED);

  // compacted layer: the per-expert tables are filled on the host before anything else
  std::vector<int32_t> count(CAMERA_MAX_EXPERTS, 17);
  EXPECT(camera_layer_forward_compact(ctx, nullptr, FAKE, CAMERA_BF16, 0, 64, 64, (int32_t*)FAKE, (float*)FAKE, 2, CAMERA_MAX_EXPERTS - 1, 1,
                                      count.data(), 64, FAKE, FAKE, FAKE, 0, (float*)FAKE) == CAMERA_OK);   // n == 0: nothing to do
  count[3] = -1;
  EXPECT(camera_layer_forward_compact(ctx, nullptr, FAKE, CAMERA_BF16, 16, 64, 64, (int32_t*)FAKE, (float*)FAKE, 2, 8, 0, count.data(), 64,
                                      FAKE, FAKE, FAKE, 0, (float*)FAKE) == CAMERA_EINVAL);
  EXPECT(camera_gather_micro_experts(ctx, nullptr, CAMERA_BF16, 8, 64, 32, FAKE, FAKE, 64 * 32, FAKE, 64 * 32, (int32_t*)FAKE, 8 * 64 + 1, 0,
                                     nullptr, 1, FAKE, FAKE, FAKE) == CAMERA_EINVAL);
  EXPECT(camera_input_channel_energy(ctx, nullptr, FAKE, CAMERA_BF16, 16, 64, 64, (int32_t*)FAKE, 9, 8, (float*)FAKE) == CAMERA_EINVAL);
  EXPECT(camera_output_error(ctx, nullptr, nullptr, nullptr, 0, 64, nullptr) == CAMERA_OK);

  double ms = 0;
  int64_t launches = 0;
  EXPECT(camera_profile_enable(ctx, 1) == CAMERA_OK);
  EXPECT(camera_profile_read(ctx, CAMERA_K_COUNT, &ms, &launches) == CAMERA_EINVAL);
  EXPECT(camera_destroy(ctx) == CAMERA_OK);
  EXPECT(camera_destroy(nullptr) == CAMERA_OK);
  if (failures) std::fprintf(stderr, "%d check(s) failed\n", failures);
  else std::printf("abi host checks: all passed\n");
  return failures ? 1 : 0;
}
