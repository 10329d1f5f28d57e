// Host-side sanitizer driver for the C ABI's argument layer.  Built by tests/test_abi_sanitized.py
// together with api.hip, both with AddressSanitizer and UndefinedBehaviorSanitizer on the host
// side; it calls every entry point with arguments that must be rejected before any HIP call and
// sweeps the workspace planner over small, real and extreme extents.  No GPU is needed.
#include <cstdio>
#include <cstring>
#include <initializer_list>
#include "pg_head.h"
static int fails = 0;
#define EXPECT(call, code) do { int32_t rc_ = (call); if (rc_ != (code)) { printf("FAIL line %d: rc=%d want %d (%s)\n", __LINE__, rc_, (code), pg_last_error()); ++fails; } } while (0)
int main() {
  pg_params p;
  memset(&p, 0, sizeof p);
  p.temperature = 1.f; p.clip_eps_lo = p.clip_eps_hi = 0.2f; p.geo_lo = 0.999f; p.geo_hi = 1.001f; p.veto_ratio = 1e-4f; p.trunc_c = 2.f;
  void* one = (void*)16;
  size_t big = (size_t)1 << 30;
  EXPECT(trloo_advantage(nullptr, (const uint8_t*)one, 1, 1, 1, 1.f, nullptr, (double*)one, nullptr, nullptr), PG_ERR_INVALID_ARG);
  EXPECT(pg_logprob_fwd(one, one, (const int32_t*)one, nullptr, 8, 64, 100, &p, (float*)one, nullptr, nullptr, one, 16, nullptr), PG_ERR_WORKSPACE_TOO_SMALL);
  EXPECT(pg_logprob_fwd(one, one, (const int32_t*)one, nullptr, 8, 72, 100, &p, (float*)one, nullptr, nullptr, one, big, nullptr), PG_ERR_UNSUPPORTED_SHAPE);
  for (int64_t T : {0ll, 1ll, 255ll, 43697ll, (1ll << 30)})
    for (int64_t V : {1ll, 1000ll, 151936ll})
      for (int dt = 0; dt < 2; ++dt) { p.dtype = dt; (void)pg_workspace_bytes(T, 5120, V, 50, &p, PG_CALL_LOSS_FWD_BWD); (void)pg_workspace_bytes(T, 64, V, 0, &p, PG_CALL_LOGPROB_FWD); }
  p.dtype = 0;
  p.mismatch_mode = 1;
  EXPECT(pg_loss_fwd_bwd(one, one, (const int32_t*)one, (const uint8_t*)one, (const int32_t*)one, 1, (const double*)one, nullptr, nullptr, (const float*)one, nullptr, 8, 64, 100, &p, (float*)one, one, one, nullptr, nullptr, nullptr, one, big, nullptr), PG_ERR_INVALID_ARG);
  p.mismatch_mode = 7;
  EXPECT(pg_sft_fwd_bwd(one, one, (const int32_t*)one, (const uint8_t*)one, 8, 64, 100, &p, (float*)one, one, one, nullptr, nullptr, nullptr, one, big, nullptr), PG_ERR_INVALID_ARG);
  p.mismatch_mode = 0;
  EXPECT(pg_head_shard_fwd(one, one, (const int32_t*)one, nullptr, 8, 64, 100, -1, &p, (float*)one, one, big, nullptr), PG_ERR_INVALID_ARG);
  EXPECT(pg_head_partials_merge((const float*)one, nullptr, (float*)one, 4, nullptr), PG_ERR_INVALID_ARG);
  EXPECT(pg_head_partials_finish(nullptr, 4, (float*)one, nullptr, nullptr, nullptr), PG_ERR_INVALID_ARG);
  EXPECT(pg_loss_shard_bwd(one, one, (const int32_t*)one, (const uint8_t*)one, (const int32_t*)one, 1, (const double*)one, nullptr, nullptr, nullptr, nullptr, nullptr, 8, 64, 100, 0, &p, (float*)one, one, 1, one, nullptr, nullptr, nullptr, one, big, nullptr), PG_ERR_INVALID_ARG);
  EXPECT(turn_reward((const uint8_t*)one, (const float*)one, (const float*)one, (const float*)one, nullptr, 4, 3.f, (float*)one, nullptr, nullptr), PG_ERR_INVALID_ARG);
  EXPECT(prs_retain((const float*)one, nullptr, 4, 0.3f, 0.f, 0, 1, (uint8_t*)one, nullptr, nullptr), PG_ERR_INVALID_ARG);
  EXPECT(pg_monitors((const float*)one, nullptr, nullptr, (const uint8_t*)one, 4, nullptr, 0, 0, nullptr, 0, 0, nullptr, one, pg_monitors_workspace_bytes(), nullptr), PG_ERR_INVALID_ARG);
  EXPECT(pg_rmsnorm_fwd(nullptr, one, 4, 64, 1e-6f, 0, one, nullptr, nullptr), PG_ERR_INVALID_ARG);
  EXPECT(pg_rmsnorm_bwd(one, one, one, 4, 64, 1e-6f, 0, one, (float*)one, one, 0, nullptr), PG_ERR_WORKSPACE_TOO_SMALL);
  EXPECT(pg_profile_read(nullptr, nullptr), PG_ERR_INVALID_ARG);
  printf(fails ? "sanitizer driver: %d FAILED\n" : "sanitizer driver: all calls rejected as expected (%d failures)\n", fails);
  return fails != 0;
}
