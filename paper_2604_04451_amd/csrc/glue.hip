// Step glue around the block stack: patch embedding of the selected tokens, the
// output head fused with the sampler update on the selected tokens, and the text
// projection. Stand-ins that close the denoising loop (the paper's sampler is
// DPM++ with default coefficients it does not list; an Euler update is used).
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

__global__ __launch_bounds__(256) void unpatch_euler_kernel(float* __restrict__ latent, const float* __restrict__ v,
                                                            const int* __restrict__ token_idx, long Ls, int C, int T,
                                                            int Hl, int Wl, int ph, int pw, float dsigma) {
  long g = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= Ls * C) return;
  long i = g / C;
  int ch = (int)(g - i * C);
  const int Wg = Wl / pw, Hg = Hl / ph;
  long n = token_idx ? (long)token_idx[i] : i;
  int wg = (int)(n % Wg), hg = (int)((n / Wg) % Hg), t = (int)(n / ((long)Wg * Hg));
  const int cell = ph * pw;
  float* dst = latent + (((long)ch * T + t) * Hl + (long)hg * ph) * Wl + (long)wg * pw;
  const float* vi = v + i * (long)(C * cell) + ch * cell;
  for (int dy = 0; dy < ph; ++dy)
    for (int dx = 0; dx < pw; ++dx) dst[(long)dy * Wl + dx] += dsigma * vi[dy * pw + dx];
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

int32_t chorus_head_update(float* latent, const float* x, int64_t Ls, const int32_t* token_idx,
                           const chorus_glue_weights* gw, const float* t_head, float dsigma, int32_t D, int32_t C,
                           int32_t T, int32_t Hl, int32_t Wl, int32_t ph, int32_t pw, void* ws, size_t ws_bytes,
                           void* stream) {
  if (Ls < 0 || C <= 0 || T <= 0 || Hl <= 0 || Wl <= 0 || ph <= 0 || pw <= 0 || D <= 0) return CHORUS_E_ARG;
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
                     (long)Ls, C, T, Hl, Wl, ph, pw, dsigma);
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
