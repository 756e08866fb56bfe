// Step glue around the block stack: patch embedding of the selected tokens, the
// output head fused with the sampler update on the selected tokens, and the text
// projection. The sampler (Sec. 4.1: DPM++, default settings) is DPM-Solver++ in
// data-prediction form on the rectified-flow path: chorus_head_update is its first-order
// step written as the Euler update, chorus_head_update_solver the multistep form with
// classifier-free guidance and the latent fusion of Eq. 6 folded into the same pass.
#include <cmath>

#include "chorus_ops.h"
#include "common.h"

namespace chorus {
namespace {

// one thread per (selected token, channel): the ph x pw cell of that channel, split
// into a bf16 head and a bf16 remainder so the K = C*ph*pw GEMM keeps fp32-level accuracy
__global__ __launch_bounds__(256) void patch_gather_kernel(const float* __restrict__ latent,
                                                           const int* __restrict__ token_idx, long Ls, int C, int T,
                                                           int Hl, int Wl, int ph, int pw, uint16_t* __restrict__ hi,
                                                           uint16_t* __restrict__ lo) {
  long g = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= Ls * C) return;
  long i = g / C;
  int ch = (int)(g - i * C);
  const int Wg = Wl / pw, Hg = Hl / ph;
  long n = token_idx ? (long)token_idx[i] : i;
  int wg = (int)(n % Wg), hg = (int)((n / Wg) % Hg), t = (int)(n / ((long)Wg * Hg));
  const int cell = ph * pw;
  const float* src = latent + (((long)ch * T + t) * Hl + (long)hg * ph) * Wl + (long)wg * pw;
  uint16_t* oh = hi + i * (long)(C * cell) + ch * cell;
  uint16_t* ol = lo + i * (long)(C * cell) + ch * cell;
  for (int dy = 0; dy < ph; ++dy)
    for (int dx = 0; dx < pw; ++dx) {
      float v = src[(long)dy * Wl + dx];
      uint16_t h = f32_to_bf16(v);
      oh[dy * pw + dx] = h;
      ol[dy * pw + dx] = f32_to_bf16(v - bf16_to_f32(h));
    }
}

// Euler update of one (selected token, channel) cell per thread, with Eq. 6 on the selected tokens when a mask is
// given: a selected token outside M_edit receives the source latent instead of the update.
__global__ __launch_bounds__(256) void unpatch_euler_kernel(float* __restrict__ latent, const float* __restrict__ v,
                                                            const int* __restrict__ token_idx, long Ls, int C, int T,
                                                            int Hl, int Wl, int ph, int pw, float dsigma,
                                                            const float* __restrict__ SL,
                                                            const uint8_t* __restrict__ mask_edit) {
  long g = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= Ls * C) return;
  long i = g / C;
  int ch = (int)(g - i * C);
  const int Wg = Wl / pw, Hg = Hl / ph;
  long n = token_idx ? (long)token_idx[i] : i;
  int wg = (int)(n % Wg), hg = (int)((n / Wg) % Hg), t = (int)(n / ((long)Wg * Hg));
  const int cell = ph * pw;
  const long base = (((long)ch * T + t) * Hl + (long)hg * ph) * Wl + (long)wg * pw;
  float* dst = latent + base;
  if (mask_edit && mask_edit[n] == 0) {
    for (int dy = 0; dy < ph; ++dy)
      for (int dx = 0; dx < pw; ++dx) dst[(long)dy * Wl + dx] = SL[base + (long)dy * Wl + dx];
    return;
  }
  const float* vi = v + i * (long)(C * cell) + ch * cell;
  for (int dy = 0; dy < ph; ++dy)
    for (int dx = 0; dx < pw; ++dx) dst[(long)dy * Wl + dx] += dsigma * vi[dy * pw + dx];
}

// Sampler update of one (selected token, channel) cell per thread, fused with the unpatchify,
// classifier-free guidance, the history of data predictions, and Eq. 6 on the selected tokens:
//   v = CFG ? vu + g (vc - vu) : vc;  x0 = x - sigma_s v;  D = c0 x0 + c1 x0_prev (tokens with history) or x0
//   x0_prev <- x0;  latent <- M_edit ? rho x + A D : SL
template <bool CFG>
__global__ __launch_bounds__(256) void unpatch_solver_kernel(float* __restrict__ latent, const float* __restrict__ vc,
                                                             const float* __restrict__ vu, float guidance,
                                                             const int* __restrict__ token_idx, long Ls, int C, int T,
                                                             int Hl, int Wl, int ph, int pw, chorus_sampler_coef cf,
                                                             float* __restrict__ x0_prev,
                                                             const uint8_t* __restrict__ hist,
                                                             const float* __restrict__ SL,
                                                             const uint8_t* __restrict__ mask_edit) {
  long g = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= Ls * C) return;
  long i = g / C;
  int ch = (int)(g - i * C);
  const int Wg = Wl / pw, Hg = Hl / ph;
  long n = token_idx ? (long)token_idx[i] : i;
  int wg = (int)(n % Wg), hg = (int)((n / Wg) % Hg), t = (int)(n / ((long)Wg * Hg));
  const int cell = ph * pw;
  const long base = (((long)ch * T + t) * Hl + (long)hg * ph) * Wl + (long)wg * pw;
  const long vrow = i * (long)(C * cell) + ch * cell;
  const bool second = cf.c1 != 0.f && (hist == nullptr || hist[n] != 0);
  const bool keep = mask_edit == nullptr || mask_edit[n] != 0;
  for (int dy = 0; dy < ph; ++dy)
    for (int dx = 0; dx < pw; ++dx) {
      const long o = base + (long)dy * Wl + dx;
      const float x = latent[o];
      float v = vc[vrow + dy * pw + dx];
      if (CFG) {
        const float u = vu[vrow + dy * pw + dx];
        v = u + guidance * (v - u);
      }
      const float x0 = x - cf.sigma_s * v;
      float d = x0;
      if (second) d = cf.c0 * x0 + cf.c1 * x0_prev[o];
      if (x0_prev) x0_prev[o] = x0;
      latent[o] = keep ? cf.rho * x + cf.A * d : SL[o];
    }
}

#define CHK(call)                       \
  do {                                  \
    int32_t st__ = (call);              \
    if (st__ != CHORUS_OK) return st__; \
  } while (0)

}  // namespace
}  // namespace chorus

using namespace chorus;

extern "C" {

size_t chorus_glue_workspace_bytes(int32_t D, int32_t P, int64_t Ls) {
  if (Ls < 1) Ls = 1;
  size_t embed = 2 * align_up((size_t)Ls * P * 2, 256);
  size_t head = align_up((size_t)Ls * D * 2, 256) + align_up((size_t)Ls * P * 4, 256);
  return embed > head ? embed : head;
}

int32_t chorus_patch_embed(const float* latent, int32_t C, int32_t T, int32_t Hl, int32_t Wl, int32_t ph, int32_t pw,
                           const int32_t* token_idx, int64_t Ls, const chorus_glue_weights* gw, int32_t D, float* x,
                           void* ws, size_t ws_bytes, void* stream) {
  if (Ls < 0 || C <= 0 || T <= 0 || Hl <= 0 || Wl <= 0 || ph <= 0 || pw <= 0 || D <= 0) return CHORUS_E_ARG;
  if (Ls == 0) return CHORUS_OK;
  if (!latent || !gw || !x || !gw->w_patch) return CHORUS_E_ARG;
  const int P = C * ph * pw;
  if (Hl % ph || Wl % pw || P % 64 || D % 8) return CHORUS_E_SHAPE;
  if (!token_idx && Ls > (int64_t)T * (Hl / ph) * (Wl / pw)) return CHORUS_E_SHAPE;
  if (!ws || ws_bytes < chorus_glue_workspace_bytes(D, P, Ls)) return CHORUS_E_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  uint16_t* hi = (uint16_t*)ws;
  uint16_t* lo = (uint16_t*)((uint8_t*)ws + align_up((size_t)Ls * P * 2, 256));
  long n = Ls * C;
  hipLaunchKernelGGL(patch_gather_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, latent, token_idx, (long)Ls,
                     C, T, Hl, Wl, ph, pw, hi, lo);
  CHORUS_LAUNCH_CHECK();
  CHK(chorus_gemm_bf16(hi, gw->w_patch, Ls, D, P, CHORUS_EPI_F32, x, gw->b_patch, nullptr, nullptr, 1.f, stream));
  CHK(chorus_gemm_bf16(lo, gw->w_patch, Ls, D, P, CHORUS_EPI_RESID, x, nullptr, nullptr, nullptr, 1.f, stream));
  return CHORUS_OK;
}

int32_t chorus_head_update_region(float* latent, const float* x, int64_t Ls, const int32_t* token_idx,
                                  const chorus_glue_weights* gw, const float* t_head, float dsigma, const float* SL,
                                  const uint8_t* mask_edit, int32_t D, int32_t C, int32_t T, int32_t Hl, int32_t Wl,
                                  int32_t ph, int32_t pw, void* ws, size_t ws_bytes, void* stream) {
  if (Ls < 0 || C <= 0 || T <= 0 || Hl <= 0 || Wl <= 0 || ph <= 0 || pw <= 0 || D <= 0) return CHORUS_E_ARG;
  if ((SL != nullptr) != (mask_edit != nullptr)) return CHORUS_E_ARG;
  if (Ls == 0) return CHORUS_OK;
  if (!latent || !x || !gw || !t_head || !gw->w_head || !gw->head_table) return CHORUS_E_ARG;
  const int P = C * ph * pw;
  if (Hl % ph || Wl % pw || P % 8 || D % 64) return CHORUS_E_SHAPE;
  if (!token_idx && Ls > (int64_t)T * (Hl / ph) * (Wl / pw)) return CHORUS_E_SHAPE;
  if (!ws || ws_bytes < chorus_glue_workspace_bytes(D, P, Ls)) return CHORUS_E_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  uint16_t* h = (uint16_t*)ws;
  float* v = (float*)((uint8_t*)ws + align_up((size_t)Ls * D * 2, 256));
  CHK(chorus_ln_modulate(x, h, Ls, D, gw->head_table + D, t_head + D, gw->head_table, t_head, 1, stream));
  CHK(chorus_gemm_bf16(h, gw->w_head, Ls, P, D, CHORUS_EPI_F32, v, gw->b_head, nullptr, nullptr, 1.f, stream));
  long n = Ls * C;
  hipLaunchKernelGGL(unpatch_euler_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, latent, v, token_idx,
                     (long)Ls, C, T, Hl, Wl, ph, pw, dsigma, SL, mask_edit);
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

int32_t chorus_head_update(float* latent, const float* x, int64_t Ls, const int32_t* token_idx,
                           const chorus_glue_weights* gw, const float* t_head, float dsigma, int32_t D, int32_t C,
                           int32_t T, int32_t Hl, int32_t Wl, int32_t ph, int32_t pw, void* ws, size_t ws_bytes,
                           void* stream) {
  return chorus_head_update_region(latent, x, Ls, token_idx, gw, t_head, dsigma, nullptr, nullptr, D, C, T, Hl, Wl, ph, pw,
                                   ws, ws_bytes, stream);
}

int32_t chorus_sampler_coefficients(const float* sigmas, int32_t n_steps, int32_t i, int32_t order,
                                    chorus_sampler_coef* out) {
  if (!sigmas || !out || n_steps < 1 || i < 0 || i >= n_steps || order < 1 || order > 2) return CHORUS_E_ARG;
  const double s = sigmas[i], t = sigmas[i + 1];
  if (!(s > 0.0 && s <= 1.0 && t >= 0.0 && t < s)) return CHORUS_E_ARG;
  const double a_s = 1.0 - s, a_t = 1.0 - t;
  double c0 = 1.0, c1 = 0.0;
  if (order == 2 && i > 0 && t > 0.0) {
    const double p = sigmas[i - 1];
    if (!(p > s && p <= 1.0)) return CHORUS_E_ARG;
    const double a_p = 1.0 - p;
    if (a_p > 0.0) {  // a history taken at sigma = 1 lies infinitely far back in lambda and has no weight
      const double lam_p = log(a_p / p), lam_s = log(a_s / s), lam_t = log(a_t / t);
      const double inv2r = (lam_t - lam_s) / (2.0 * (lam_s - lam_p));
      c0 = 1.0 + inv2r;
      c1 = -inv2r;
    }
  }
  out->sigma_s = (float)s;
  out->rho = (float)(t / s);
  out->A = (float)(a_t - t * a_s / s);
  out->c0 = (float)c0;
  out->c1 = (float)c1;
  return CHORUS_OK;
}

size_t chorus_head_solver_workspace_bytes(int32_t D, int32_t P, int64_t Ls, int32_t cfg) {
  if (Ls < 1) Ls = 1;
  return align_up((size_t)Ls * D * 2, 256) + (cfg ? 2 : 1) * align_up((size_t)Ls * P * 4, 256);
}

int32_t chorus_head_update_solver(float* latent, const float* x, const float* x_uncond, float guidance, int64_t Ls,
                                  const int32_t* token_idx, const chorus_glue_weights* gw, const float* t_head,
                                  const chorus_sampler_coef* coef, float* x0_prev, const uint8_t* hist, const float* SL,
                                  const uint8_t* mask_edit, int32_t D, int32_t C, int32_t T, int32_t Hl, int32_t Wl,
                                  int32_t ph, int32_t pw, void* ws, size_t ws_bytes, void* stream) {
  if (Ls < 0 || C <= 0 || T <= 0 || Hl <= 0 || Wl <= 0 || ph <= 0 || pw <= 0 || D <= 0) return CHORUS_E_ARG;
  if (!coef || (coef->c1 != 0.f && !x0_prev) || ((mask_edit != nullptr) != (SL != nullptr))) return CHORUS_E_ARG;
  if (Ls == 0) return CHORUS_OK;
  if (!latent || !x || !gw || !t_head || !gw->w_head || !gw->head_table) return CHORUS_E_ARG;
  if (x0_prev == latent || (SL && (SL == latent || SL == x0_prev))) return CHORUS_E_ARG;
  const int P = C * ph * pw;
  if (Hl % ph || Wl % pw || P % 8 || D % 64) return CHORUS_E_SHAPE;
  if (!token_idx && Ls > (int64_t)T * (Hl / ph) * (Wl / pw)) return CHORUS_E_SHAPE;
  const int cfg = x_uncond != nullptr;
  if (!ws || ws_bytes < chorus_head_solver_workspace_bytes(D, P, Ls, cfg)) return CHORUS_E_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  uint16_t* h = (uint16_t*)ws;
  float* v = (float*)((uint8_t*)ws + align_up((size_t)Ls * D * 2, 256));
  float* vu = (float*)((uint8_t*)v + align_up((size_t)Ls * P * 4, 256));
  CHK(chorus_ln_modulate(x, h, Ls, D, gw->head_table + D, t_head + D, gw->head_table, t_head, 1, stream));
  CHK(chorus_gemm_bf16(h, gw->w_head, Ls, P, D, CHORUS_EPI_F32, v, gw->b_head, nullptr, nullptr, 1.f, stream));
  if (cfg) {
    CHK(chorus_ln_modulate(x_uncond, h, Ls, D, gw->head_table + D, t_head + D, gw->head_table, t_head, 1, stream));
    CHK(chorus_gemm_bf16(h, gw->w_head, Ls, P, D, CHORUS_EPI_F32, vu, gw->b_head, nullptr, nullptr, 1.f, stream));
  }
  long n = Ls * C;
  dim3 grid((unsigned)((n + 255) / 256));
  if (cfg)
    hipLaunchKernelGGL(unpatch_solver_kernel<true>, grid, dim3(256), 0, s, latent, v, vu, guidance, token_idx, (long)Ls, C, T,
                       Hl, Wl, ph, pw, *coef, x0_prev, hist, SL, mask_edit);
  else
    hipLaunchKernelGGL(unpatch_solver_kernel<false>, grid, dim3(256), 0, s, latent, v, (const float*)nullptr, 1.f, token_idx,
                       (long)Ls, C, T, Hl, Wl, ph, pw, *coef, x0_prev, hist, SL, mask_edit);
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

size_t chorus_text_project_workspace_bytes(int32_t Lt, int32_t D) {
  return align_up((size_t)(Lt > 0 ? Lt : 1) * (size_t)(D > 0 ? D : 1) * 2, 256);
}

int32_t chorus_text_project(const uint16_t* text, int32_t Lt, int32_t text_dim, int32_t D, const uint16_t* w1,
                            const float* b1, const uint16_t* w2, const float* b2, uint16_t* ctx, void* ws,
                            size_t ws_bytes, void* stream) {
  if (Lt < 0 || text_dim <= 0 || D <= 0) return CHORUS_E_ARG;
  if (Lt == 0) return CHORUS_OK;
  if (!text || !w1 || !w2 || !ctx) return CHORUS_E_ARG;
  if (text_dim % 64 || D % 64) return CHORUS_E_SHAPE;
  if (!ws || ws_bytes < chorus_text_project_workspace_bytes(Lt, D)) return CHORUS_E_WORKSPACE;
  uint16_t* hid = (uint16_t*)ws;
  CHK(chorus_gemm_bf16(text, w1, Lt, D, text_dim, CHORUS_EPI_GELU_BF16, hid, b1, nullptr, nullptr, 1.f, stream));
  CHK(chorus_gemm_bf16(hid, w2, Lt, D, D, CHORUS_EPI_BF16, ctx, b2, nullptr, nullptr, 1.f, stream));
  return CHORUS_OK;
}

}  // extern "C"
