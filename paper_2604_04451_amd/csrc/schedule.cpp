// Stage boundaries (Eq. 1) and the TGAA decay (Eq. 4): host-only scalar code.
#include <cmath>

#include "chorus.h"

namespace {
inline double clampd(double v, double lo, double hi) { return v < lo ? lo : (v > hi ? hi : v); }
inline int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }
}  // namespace

namespace {
int32_t schedule_impl(float m, float tau, int32_t N, const chorus_sched_params* params, const int32_t* stored_steps,
                      int32_t n_stored, int32_t* K1, int32_t* K2, int32_t* slot, chorus_step_plan* plan);
}

extern "C" int32_t chorus_denoise_schedule(float m, float tau, int32_t N, const chorus_sched_params* params,
                                           int32_t* K1, int32_t* K2, chorus_step_plan* plan) {
  return schedule_impl(m, tau, N, params, nullptr, -1, K1, K2, nullptr, plan);
}

extern "C" int32_t chorus_denoise_schedule_stored(float m, float tau, int32_t N, const chorus_sched_params* params,
                                                  const int32_t* stored_steps, int32_t n_stored, int32_t* K1,
                                                  int32_t* K2, int32_t* slot, chorus_step_plan* plan) {
  if (n_stored < 0 || (n_stored > 0 && !stored_steps)) return CHORUS_E_ARG;
  return schedule_impl(m, tau, N, params, stored_steps, n_stored, K1, K2, slot, plan);
}

namespace {
int32_t schedule_impl(float m, float tau, int32_t N, const chorus_sched_params* params, const int32_t* stored_steps,
                      int32_t n_stored, int32_t* K1, int32_t* K2, int32_t* slot, chorus_step_plan* plan) {
  if (slot) *slot = -1;
  if (N < 0 || (N > 0 && !plan)) return CHORUS_E_ARG;
  chorus_sched_params p;
  if (params) {
    p = *params;
  } else {
    p.a1 = p.b1 = p.a2 = p.b2 = 0.25;
    p.r3 = 1;
    p.Gamma_k = p.Gamma_o = 1.5;
    p.lam = 0.5;
    p.gamma_override = 0.0;
  }
  if (p.r3 < 0) return CHORUS_E_ARG;
  // the fallback rule is "m < tau"; a NaN score is a miss as well
  if (!(m >= tau)) {
    for (int i = 0; i < N; ++i) plan[i] = chorus_step_plan{3, 1.0f, 1.0f};
    if (K1) *K1 = 0;
    if (K2) *K2 = 0;
    return CHORUS_OK;
  }
  const double dm = (double)m, dt = (double)tau;
  const double s = dt < 1.0 ? clampd((dm - dt) / (1.0 - dt), 0.0, 1.0) : 1.0;
  const int hi = N - p.r3 > 0 ? N - p.r3 : 0;
  int k1 = clampi((int)std::floor(N * (p.a1 + p.b1 * s) + 1e-9), 0, hi);
  if (n_stored >= 0) {
    // full reuse resumes from a stored state: the deepest one not beyond Eq. 1's K1, else the request runs as a miss
    int best = 0, best_slot = -1;
    for (int j = 0; j < n_stored; ++j)
      if (stored_steps[j] >= 1 && stored_steps[j] <= k1 && stored_steps[j] > best) {
        best = stored_steps[j];
        best_slot = j;
      }
    if (best_slot < 0) {
      for (int i = 0; i < N; ++i) plan[i] = chorus_step_plan{3, 1.0f, 1.0f};
      if (K1) *K1 = 0;
      if (K2) *K2 = 0;
      return CHORUS_OK;
    }
    k1 = best;
    if (slot) *slot = best_slot;
  }
  const int k2 = clampi(k1 + (int)std::floor(N * (p.a2 + p.b2 * s) + 1e-9), k1, hi);
  for (int i = 0; i < N; ++i) {
    if (i < k1) {
      plan[i] = chorus_step_plan{1, 1.0f, 1.0f};
      continue;
    }
    const int stage = i < k2 ? 2 : 3;
    const int span = k2 - k1 > 1 ? k2 - k1 : 1;
    double w = 1.0 - (double)(i - k1) / (double)span;
    if (w < 0.0) w = 0.0;
    double gk = 1.0 + (p.Gamma_k - 1.0) * (1.0 - p.lam * s) * w;
    double go = 1.0 + (p.Gamma_o - 1.0) * (1.0 - p.lam * s) * w;
    if (gk < 1.0) gk = 1.0;
    if (go < 1.0) go = 1.0;
    if (stage == 2 && p.gamma_override > 0.0) gk = go = p.gamma_override;
    plan[i] = chorus_step_plan{stage, (float)gk, (float)go};
  }
  if (K1) *K1 = k1;
  if (K2) *K2 = k2;
  return CHORUS_OK;
}
}  // namespace
