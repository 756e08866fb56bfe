// Host-side driver for the sanitizer build of the library (AddressSanitizer + UndefinedBehaviorSanitizer on the
// host code only): walks the host-only entry points over their whole argument range and every entry point's
// argument validation and workspace sizing, none of which touches a GPU. Exits 0 when every call returned what
// it should; the sanitizers abort the process on any finding.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <limits>
#include <vector>

#include "chorus.h"
#include "chorus_ops.h"

static int failures = 0;
#define EXPECT(cond)                                                      \
  do {                                                                    \
    if (!(cond)) {                                                        \
      std::fprintf(stderr, "line %d: %s\n", __LINE__, #cond);             \
      ++failures;                                                         \
    }                                                                     \
  } while (0)

static void* fake(uintptr_t a) { return reinterpret_cast<void*>(a); }  // never dereferenced by a validation path

static void schedules() {
  const float ms[] = {-1.f, 0.f, 0.3f, 0.7499f, 0.75f, 0.8f, 0.95f, 1.f, 1.5f, std::numeric_limits<float>::quiet_NaN(),
                      std::numeric_limits<float>::infinity(), -std::numeric_limits<float>::infinity()};
  chorus_sched_params custom{0.1, 0.5, 0.2, 0.3, 2, 2.0, 1.5, 0.9, 0.0};
  chorus_sched_params over{0.25, 0.25, 0.25, 0.25, 0, 1.5, 1.5, 0.5, 1.5};
  const chorus_sched_params* ps[] = {nullptr, &custom, &over};
  for (int N : {0, 1, 2, 4, 8, 50, 64, 1000}) {
    std::vector<chorus_step_plan> plan((size_t)N);  // exactly N entries: an overrun is a heap-buffer-overflow
    for (float m : ms)
      for (const chorus_sched_params* p : ps) {
        int32_t k1 = -9, k2 = -9, slot = -9;
        EXPECT(chorus_denoise_schedule(m, 0.75f, N, p, &k1, &k2, N ? plan.data() : nullptr) == CHORUS_OK);
        EXPECT(0 <= k1 && k1 <= k2 && k2 <= N);
        for (int i = 0; i < N; ++i) EXPECT(plan[i].stage == (i < k1 ? 1 : i < k2 ? 2 : 3) && plan[i].gamma_k >= 1.f);
        EXPECT(chorus_denoise_schedule(m, 0.75f, N, p, nullptr, nullptr, N ? plan.data() : nullptr) == CHORUS_OK);
        const int32_t stored[] = {3, 1, 40, 2};
        for (int ns : {0, 1, 4}) {
          EXPECT(chorus_denoise_schedule_stored(m, 0.75f, N, p, ns ? stored : nullptr, ns, &k1, &k2, &slot,
                                                N ? plan.data() : nullptr) == CHORUS_OK);
          EXPECT(0 <= k1 && k1 <= k2 && k2 <= N && slot >= -1 && slot < (ns ? ns : 1));
          if (slot >= 0) EXPECT(stored[slot] == k1);
        }
      }
  }
  chorus_step_plan one;
  EXPECT(chorus_denoise_schedule(0.9f, 0.75f, -1, nullptr, nullptr, nullptr, &one) == CHORUS_E_ARG);
  EXPECT(chorus_denoise_schedule(0.9f, 0.75f, 3, nullptr, nullptr, nullptr, nullptr) == CHORUS_E_ARG);
  EXPECT(chorus_denoise_schedule_stored(0.9f, 0.75f, 1, nullptr, nullptr, 2, nullptr, nullptr, nullptr, &one) == CHORUS_E_ARG);
  chorus_sched_params neg = custom;
  neg.r3 = -1;
  EXPECT(chorus_denoise_schedule(0.9f, 0.75f, 1, &neg, nullptr, nullptr, &one) == CHORUS_E_ARG);
}

static void sampler() {
  for (int n : {1, 2, 4, 8, 50}) {
    std::vector<float> sig((size_t)n + 1);
    for (int i = 0; i <= n; ++i) {
      const double u = 1.0 - (double)i / n;
      sig[i] = (float)(3.0 * u / (1.0 + 2.0 * u));
    }
    for (int order : {1, 2})
      for (int i = 0; i < n; ++i) {
        chorus_sampler_coef c;
        EXPECT(chorus_sampler_coefficients(sig.data(), n, i, order, &c) == CHORUS_OK);
        EXPECT(std::isfinite(c.rho) && std::isfinite(c.A) && std::isfinite(c.c0) && std::isfinite(c.c1));
      }
    chorus_sampler_coef c;
    EXPECT(chorus_sampler_coefficients(sig.data(), n, n, 1, &c) == CHORUS_E_ARG);
    EXPECT(chorus_sampler_coefficients(sig.data(), n, -1, 1, &c) == CHORUS_E_ARG);
    EXPECT(chorus_sampler_coefficients(sig.data(), n, 0, 3, &c) == CHORUS_E_ARG);
    EXPECT(chorus_sampler_coefficients(nullptr, n, 0, 1, &c) == CHORUS_E_ARG);
  }
}

static void sizes_and_validation() {
  void* p16 = fake(16);
  chorus_lookup_result lr;
  // workspace sizes (the carving arithmetic runs on a null base)
  EXPECT(chorus_cache_lookup_workspace_bytes(0) >= 256 && chorus_cache_lookup_workspace_bytes(1 << 20) > 256);
  EXPECT(chorus_cache_lookup_batch_workspace_bytes(4096, 4096, 33) > 0);
  EXPECT(chorus_cache_lookup_lowprec_workspace_bytes(4096) >= 4096 * 4);
  EXPECT(chorus_region_compact_workspace_bytes(75600) > 0);
  chorus_block_shape bs{1536, 12, 128, 8960, 512, 21, 30, 52};
  chorus_block_shape bad{1536, 12, 96, 8960, 512, 21, 30, 52};
  EXPECT(chorus_dit_block_workspace_bytes(&bs, 32760) > chorus_dit_block_workspace_bytes(&bs, 13104));
  EXPECT(chorus_dit_block_workspace_bytes(&bad, 10) == 0 && chorus_dit_block_workspace_bytes(nullptr, 10) == 0);
  EXPECT(chorus_text_kv_bytes(&bs) > 0 && chorus_text_kv_workspace_bytes(&bs) > 0);
  chorus_model_shape ms{bs, 16, 21, 60, 104, 2, 2, 30};
  EXPECT(chorus_denoise_step_workspace_bytes(&ms, 32760) > 0);
  EXPECT(chorus_denoise_step_solver_workspace_bytes(&ms, 32760, 1) >= chorus_denoise_step_solver_workspace_bytes(&ms, 32760, 0));
  EXPECT(chorus_denoise_run_workspace_bytes(&ms, 4096) > chorus_denoise_step_workspace_bytes(&ms, 32760));
  EXPECT(chorus_model_text_kv_bytes(&ms) == 30 * chorus_text_kv_bytes(&bs));
  EXPECT(chorus_glue_workspace_bytes(1536, 64, 32760) > 0 && chorus_head_solver_workspace_bytes(1536, 64, 32760, 1) > 0);
  EXPECT(chorus_time_mod_workspace_bytes(1536, 256) > 0 && chorus_text_project_workspace_bytes(512, 1536) > 0);
  EXPECT(chorus_mfma_ceiling_workspace_bytes() > 0);
  EXPECT(chorus_mask_pooled_extent(81, 4, 1) == 21 && chorus_mask_pooled_extent(5, 0, 0) < 0 && chorus_mask_pooled_extent(5, 2, 6) < 0);
  EXPECT(chorus_cache_lowprec_bytes(10, 64, CHORUS_LP_BF16) == 1280);
  // argument validation: every call returns before any device work
  EXPECT(chorus_cache_lookup((const float*)p16, 4, 6, (const float*)p16, 0.5f, &lr, p16, 1024, nullptr) == CHORUS_E_SHAPE);
  EXPECT(chorus_cache_lookup((const float*)p16, 4, 8, (const float*)p16, 0.5f, &lr, nullptr, 0, nullptr) == CHORUS_E_WORKSPACE);
  EXPECT(chorus_cache_lookup((const float*)fake(8), 4, 8, (const float*)p16, 0.5f, &lr, p16, 1024, nullptr) == CHORUS_E_ARG);
  EXPECT(chorus_cache_lookup_static((const float*)p16, -1, 8, (const float*)p16, 0.5f, &lr, nullptr) == CHORUS_E_ARG);
  EXPECT(chorus_cache_lookup_lowprec((const float*)p16, p16, 5, 4, 64, (const float*)p16, 0.5f, &lr, nullptr, p16, 1 << 20, nullptr) == CHORUS_E_ARG);
  EXPECT(chorus_cache_lowprec_store((const float*)p16, 4, 24, CHORUS_LP_FP8, p16, nullptr) == CHORUS_E_SHAPE);
  EXPECT(chorus_cache_insert((float*)p16, (float*)p16, 4, 4, 8, 16, (const float*)p16, (const float*)p16, nullptr) == CHORUS_E_ARG);
  EXPECT(chorus_region_blend((float*)p16, (const float*)p16, (const float*)p16, (const uint8_t*)p16, 1, 1, 3, 4, 2, 2, nullptr) == CHORUS_E_SHAPE);
  EXPECT(chorus_region_blend(nullptr, nullptr, nullptr, nullptr, 0, 1, 4, 4, 2, 2, nullptr) == CHORUS_OK);
  chorus_block_weights w{};
  EXPECT(chorus_dit_block_step(&bad, &w, (float*)p16, 4, nullptr, (const uint16_t*)p16, (const float*)p16, nullptr, 1.f, p16, 1 << 20, nullptr) == CHORUS_E_SHAPE);
  const size_t need = chorus_dit_block_workspace_bytes(&bs, 256);
  EXPECT(chorus_dit_block_step(&bs, &w, (float*)p16, 256, nullptr, (const uint16_t*)p16, (const float*)p16, nullptr, 1.f, fake(256), need - 1, nullptr) == CHORUS_E_WORKSPACE);
  EXPECT(chorus_dit_block_step(&bs, &w, (float*)p16, 0, nullptr, (const uint16_t*)p16, (const float*)p16, nullptr, 1.f, nullptr, 0, nullptr) == CHORUS_OK);
  EXPECT(chorus_gemm_bf16((const uint16_t*)p16, (const uint16_t*)p16, 8, 64, 100, 0, p16, nullptr, nullptr, nullptr, 1.f, nullptr) == CHORUS_E_SHAPE);
  EXPECT(chorus_gemm_bf16_kernel((const uint16_t*)p16, (const uint16_t*)p16, 8, 64, 64, 0, p16, nullptr, nullptr, nullptr, 1.f, 9, nullptr) == CHORUS_E_ARG);
  EXPECT(chorus_attention((const uint16_t*)p16, (const uint16_t*)p16, (const uint16_t*)p16, (uint16_t*)p16, nullptr, 8, 8, 64, 64, 2, 96, 0, nullptr) == CHORUS_E_SHAPE);
  EXPECT(chorus_attention((const uint16_t*)p16, (const uint16_t*)p16, (const uint16_t*)p16, (uint16_t*)p16, nullptr, 8, 8, 64, 64, 2, 64, 2, nullptr) == CHORUS_E_ARG);
  // the run: a request the validation must refuse before the lookup is launched
  chorus_glue_weights gw{};
  chorus_run_result rr;
  std::vector<float> sig(66);
  for (int i = 0; i < 66; ++i) sig[i] = 1.f - i / 65.f;
  chorus_request rq{};
  rq.cache_emb = (float*)p16;
  rq.cache_latents = (float*)p16;
  rq.cache_N = 4;
  rq.cache_d = 8;
  rq.query = (const float*)p16;
  rq.tau = 0.75f;
  rq.n_steps = 65;
  rq.sigmas = sig.data();
  rq.t_mods = (const float*)p16;
  rq.t_heads = (const float*)p16;
  rq.text_ctx = (const uint16_t*)p16;
  rq.store_slot = -1;
  rq.solver_order = 1;
  EXPECT(chorus_denoise_run(&ms, nullptr, &gw, &rq, (float*)p16, &rr, fake(256), (size_t)1 << 40, nullptr) == CHORUS_E_SHAPE);
  rq.n_steps = 4;
  rq.solver_order = 3;
  EXPECT(chorus_denoise_run(&ms, nullptr, &gw, &rq, (float*)p16, &rr, fake(256), (size_t)1 << 40, nullptr) == CHORUS_E_ARG);
  rq.solver_order = 1;
  EXPECT(chorus_denoise_run(&ms, nullptr, &gw, &rq, (float*)p16, &rr, fake(256), 1024, nullptr) == CHORUS_E_WORKSPACE);
  const int32_t depths[] = {1, 1};
  rq.latent_steps = depths;
  rq.n_latent_steps = 2;
  EXPECT(chorus_denoise_run(&ms, nullptr, &gw, &rq, (float*)p16, &rr, fake(256), (size_t)1 << 40, nullptr) == CHORUS_E_ARG);
  const int32_t r0[3] = {0, 1, 1}, r1[3] = {1, 3, 3}, rbad[3] = {0, 0, 0};
  EXPECT(chorus_mask_hierarchy((const uint8_t*)p16, 21, 30, 52, r1, rbad, (uint8_t*)fake(4096), (uint8_t*)fake(8192), nullptr) == CHORUS_E_ARG);
  EXPECT(chorus_mask_hierarchy(nullptr, 21, 30, 52, r0, r1, (uint8_t*)fake(4096), (uint8_t*)fake(8192), nullptr) == CHORUS_E_ARG);
  EXPECT(chorus_mask_project((const uint8_t*)p16, 21, nullptr, 81, 480, 832, 4, 16, 16, 1, (uint8_t*)fake(1 << 20), nullptr) == CHORUS_E_ARG);
}

int main() {
  schedules();
  sampler();
  sizes_and_validation();
  if (failures) {
    std::fprintf(stderr, "%d expectation(s) failed\n", failures);
    return 1;
  }
  std::puts("sanitize_driver: ok");
  return 0;
}
