// chorus_denoise_step: one computed denoising step (stage 2 or stage 3) as one
// host call: patch-embed the selected tokens, run every block on them, apply the
// head + sampler update to them, and (stage 2) fuse with the source latent (Eq. 6).
#include "chorus_ops.h"
#include "common.h"

using namespace chorus;

namespace {
struct StepWs {
  float* x;
  void* glue;
  size_t glue_bytes;
  void* block;
  size_t block_bytes;
  size_t bytes;
};

StepWs carve_step(const chorus_model_shape& m, long Ls, void* base) {
  StepWs w;
  const BytePtr p(base);
  size_t off = 0;
  const long rows = Ls > 0 ? Ls : 1;
  w.x = (float*)(p + off);
  off += align_up((size_t)rows * m.block.D * 4, 256);
  w.glue = p + off;
  w.glue_bytes = chorus_glue_workspace_bytes(m.block.D, m.C * m.ph * m.pw, rows);
  off += align_up(w.glue_bytes, 256);
  w.block = p + off;
  w.block_bytes = chorus_dit_block_workspace_bytes(&m.block, rows);
  off += align_up(w.block_bytes, 256);
  w.bytes = off;
  return w;
}

int32_t check_model(const chorus_model_shape* m) {
  if (!m) return CHORUS_E_ARG;
  if (m->C <= 0 || m->T <= 0 || m->Hl <= 0 || m->Wl <= 0 || m->ph <= 0 || m->pw <= 0 || m->n_blocks < 0)
    return CHORUS_E_SHAPE;
  if (m->Hl % m->ph || m->Wl % m->pw) return CHORUS_E_SHAPE;
  if (m->block.gT != m->T || m->block.gH != m->Hl / m->ph || m->block.gW != m->Wl / m->pw) return CHORUS_E_SHAPE;
  if (chorus_dit_block_workspace_bytes(&m->block, 1) == 0) return CHORUS_E_SHAPE;
  return CHORUS_OK;
}
}  // namespace

extern "C" {

size_t chorus_denoise_step_workspace_bytes(const chorus_model_shape* model, int64_t Ls) {
  if (check_model(model) != CHORUS_OK || Ls < 0) return 0;
  return carve_step(*model, Ls, nullptr).bytes;
}

}  // extern "C"

namespace {
// one computed step; the prompt enters either as text_ctx (K / V projected inside every block) or as text_kv, the
// per-block projections made once per request by chorus_text_kv_project (block b at text_kv + b * chorus_text_kv_bytes)
int32_t denoise_step_impl(const chorus_model_shape* model, const chorus_block_weights* blocks, const chorus_glue_weights* gw,
                          float* latent, const int32_t* token_idx, int64_t Ls, const uint16_t* text_ctx,
                          const uint8_t* text_kv, const float* t_mod, const float* t_head, const float* tgaa_key_scale,
                          float gamma_o, float dsigma, const float* SL, const uint8_t* mask_edit, bool outside_is_source,
                          void* ws, size_t ws_bytes, void* stream) {
  int32_t st = check_model(model);
  if (st != CHORUS_OK) return st;
  const chorus_model_shape& m = *model;
  const int64_t Ltok = (int64_t)m.T * (m.Hl / m.ph) * (m.Wl / m.pw);
  if (Ls < 0 || Ls > Ltok) return CHORUS_E_ARG;
  if (!token_idx && Ls != Ltok) return CHORUS_E_ARG;
  if (!latent || !gw || (!text_ctx && !text_kv) || !t_mod || !t_head || (m.n_blocks > 0 && !blocks)) return CHORUS_E_ARG;
  if ((mask_edit != nullptr) != (SL != nullptr)) return CHORUS_E_ARG;
  if (!ws) return CHORUS_E_WORKSPACE;
  StepWs w = carve_step(m, Ls, ws);
  if (ws_bytes < w.bytes) return CHORUS_E_WORKSPACE;
  if (Ls > 0) {
    st = chorus_patch_embed(latent, m.C, m.T, m.Hl, m.Wl, m.ph, m.pw, token_idx, Ls, gw, m.block.D, w.x, w.glue,
                            w.glue_bytes, stream);
    if (st != CHORUS_OK) return st;
    const size_t kv_bytes = chorus_text_kv_bytes(&m.block);
    for (int b = 0; b < m.n_blocks; ++b) {
      if (text_kv)
        st = chorus_dit_block_step_kv(&m.block, &blocks[b], w.x, Ls, token_idx, (const uint16_t*)(text_kv + b * kv_bytes),
                                      t_mod, tgaa_key_scale, gamma_o, w.block, w.block_bytes, stream);
      else
        st = chorus_dit_block_step(&m.block, &blocks[b], w.x, Ls, token_idx, text_ctx, t_mod, tgaa_key_scale, gamma_o,
                                   w.block, w.block_bytes, stream);
      if (st != CHORUS_OK) return st;
    }
    // Eq. 6 inside the update pass when the latent outside the selection already is the source latent
    const bool fused = mask_edit && outside_is_source;
    st = chorus_head_update_region(latent, w.x, Ls, token_idx, gw, t_head, dsigma, fused ? SL : nullptr,
                                   fused ? mask_edit : nullptr, m.block.D, m.C, m.T, m.Hl, m.Wl, m.ph, m.pw, w.glue,
                                   w.glue_bytes, stream);
    if (st != CHORUS_OK) return st;
  }
  if (mask_edit && !outside_is_source) {
    st = chorus_region_blend(latent, latent, SL, mask_edit, m.C, m.T, m.Hl, m.Wl, m.ph, m.pw, stream);
    if (st != CHORUS_OK) return st;
  }
  return CHORUS_OK;
}
}  // namespace

namespace {
struct SolverWs {
  float* x;
  float* xu;
  void* glue;
  size_t glue_bytes;
  void* block;
  size_t block_bytes;
  size_t bytes;
};

SolverWs carve_solver(const chorus_model_shape& m, long Ls, int cfg, void* base) {
  SolverWs w;
  const BytePtr p(base);
  size_t off = 0;
  const long rows = Ls > 0 ? Ls : 1;
  const int P = m.C * m.ph * m.pw;
  w.x = (float*)(p + off);
  off += align_up((size_t)rows * m.block.D * 4, 256);
  w.xu = nullptr;
  if (cfg) {
    w.xu = (float*)(p + off);
    off += align_up((size_t)rows * m.block.D * 4, 256);
  }
  w.glue = p + off;
  const size_t embed = chorus_glue_workspace_bytes(m.block.D, P, rows);
  const size_t head = chorus_head_solver_workspace_bytes(m.block.D, P, rows, cfg);
  w.glue_bytes = embed > head ? embed : head;
  off += align_up(w.glue_bytes, 256);
  w.block = p + off;
  w.block_bytes = chorus_dit_block_workspace_bytes(&m.block, rows);
  off += align_up(w.block_bytes, 256);
  w.bytes = off;
  return w;
}

int32_t device_copy(float* dst, const float* src, long n, hipStream_t s);
}  // namespace

extern "C" {

size_t chorus_denoise_step_solver_workspace_bytes(const chorus_model_shape* model, int64_t Ls, int32_t cfg) {
  if (check_model(model) != CHORUS_OK || Ls < 0) return 0;
  return carve_solver(*model, Ls, cfg != 0, nullptr).bytes;
}

int32_t chorus_denoise_step_solver(const chorus_model_shape* model, const chorus_block_weights* blocks,
                                   const chorus_glue_weights* gw, float* latent, const int32_t* token_idx, int64_t Ls,
                                   const void* text_kv, const void* text_kv_uncond, float guidance, const float* t_mod,
                                   const float* t_head, const float* tgaa_key_scale, float gamma_o,
                                   const chorus_sampler_coef* coef, float* x0_prev, const uint8_t* hist, const float* SL,
                                   const uint8_t* mask_edit, int32_t outside_is_source, void* ws, size_t ws_bytes,
                                   void* stream) {
  int32_t st = check_model(model);
  if (st != CHORUS_OK) return st;
  const chorus_model_shape& m = *model;
  const int64_t Ltok = (int64_t)m.T * (m.Hl / m.ph) * (m.Wl / m.pw);
  if (Ls < 0 || Ls > Ltok) return CHORUS_E_ARG;
  if (!token_idx && Ls != Ltok) return CHORUS_E_ARG;
  if (!latent || !gw || !t_mod || !t_head || !coef || (m.n_blocks > 0 && (!blocks || !text_kv))) return CHORUS_E_ARG;
  if ((mask_edit != nullptr) != (SL != nullptr)) return CHORUS_E_ARG;
  if (coef->c1 != 0.f && !x0_prev) return CHORUS_E_ARG;
  if (!ws) return CHORUS_E_WORKSPACE;
  const int cfg = text_kv_uncond != nullptr;
  SolverWs w = carve_solver(m, Ls, cfg, ws);
  if (ws_bytes < w.bytes) return CHORUS_E_WORKSPACE;
  if (Ls > 0) {
    st = chorus_patch_embed(latent, m.C, m.T, m.Hl, m.Wl, m.ph, m.pw, token_idx, Ls, gw, m.block.D, w.x, w.glue,
                            w.glue_bytes, stream);
    if (st != CHORUS_OK) return st;
    if (cfg) {
      st = device_copy(w.xu, w.x, (long)Ls * m.block.D, (hipStream_t)stream);
      if (st != CHORUS_OK) return st;
    }
    const size_t kv_bytes = chorus_text_kv_bytes(&m.block);
    for (int b = 0; b < m.n_blocks; ++b) {
      st = chorus_dit_block_step_kv(&m.block, &blocks[b], w.x, Ls, token_idx,
                                    (const uint16_t*)((const uint8_t*)text_kv + b * kv_bytes), t_mod, tgaa_key_scale,
                                    gamma_o, w.block, w.block_bytes, stream);
      if (st != CHORUS_OK) return st;
    }
    for (int b = 0; cfg && b < m.n_blocks; ++b) {
      st = chorus_dit_block_step_kv(&m.block, &blocks[b], w.xu, Ls, token_idx,
                                    (const uint16_t*)((const uint8_t*)text_kv_uncond + b * kv_bytes), t_mod, nullptr, 1.f,
                                    w.block, w.block_bytes, stream);
      if (st != CHORUS_OK) return st;
    }
    st = chorus_head_update_solver(latent, w.x, w.xu, guidance, Ls, token_idx, gw, t_head, coef, x0_prev, hist, SL,
                                   mask_edit, m.block.D, m.C, m.T, m.Hl, m.Wl, m.ph, m.pw, w.glue, w.glue_bytes, stream);
    if (st != CHORUS_OK) return st;
  }
  if (mask_edit && !outside_is_source) {
    st = chorus_region_blend(latent, latent, SL, mask_edit, m.C, m.T, m.Hl, m.Wl, m.ph, m.pw, stream);
    if (st != CHORUS_OK) return st;
  }
  return CHORUS_OK;
}

int32_t chorus_denoise_step(const chorus_model_shape* model, const chorus_block_weights* blocks,
                            const chorus_glue_weights* gw, float* latent, const int32_t* token_idx, int64_t Ls,
                            const uint16_t* text_ctx, const float* t_mod, const float* t_head,
                            const float* tgaa_key_scale, float gamma_o, float dsigma, const float* SL,
                            const uint8_t* mask_edit, void* ws, size_t ws_bytes, void* stream) {
  if (!text_ctx) return CHORUS_E_ARG;
  return denoise_step_impl(model, blocks, gw, latent, token_idx, Ls, text_ctx, nullptr, t_mod, t_head, tgaa_key_scale,
                           gamma_o, dsigma, SL, mask_edit, false, ws, ws_bytes, stream);
}

int32_t chorus_denoise_step_kv(const chorus_model_shape* model, const chorus_block_weights* blocks,
                               const chorus_glue_weights* gw, float* latent, const int32_t* token_idx, int64_t Ls,
                               const void* text_kv, const float* t_mod, const float* t_head,
                               const float* tgaa_key_scale, float gamma_o, float dsigma, const float* SL,
                               const uint8_t* mask_edit, void* ws, size_t ws_bytes, void* stream) {
  if (!text_kv) return CHORUS_E_ARG;
  return denoise_step_impl(model, blocks, gw, latent, token_idx, Ls, nullptr, (const uint8_t*)text_kv, t_mod, t_head,
                           tgaa_key_scale, gamma_o, dsigma, SL, mask_edit, false, ws, ws_bytes, stream);
}

size_t chorus_model_text_kv_bytes(const chorus_model_shape* model) {
  if (check_model(model) != CHORUS_OK) return 0;
  return (size_t)model->n_blocks * chorus_text_kv_bytes(&model->block);
}

int32_t chorus_model_text_kv_project(const chorus_model_shape* model, const chorus_block_weights* blocks,
                                     const uint16_t* text_ctx, void* text_kv, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = check_model(model);
  if (st != CHORUS_OK) return st;
  if (model->n_blocks == 0) return CHORUS_OK;
  if (!blocks || !text_ctx || !text_kv) return CHORUS_E_ARG;
  const size_t kv_bytes = chorus_text_kv_bytes(&model->block);
  for (int b = 0; b < model->n_blocks; ++b) {
    st = chorus_text_kv_project(&model->block, &blocks[b], text_ctx, (uint16_t*)((uint8_t*)text_kv + b * kv_bytes), ws,
                                ws_bytes, stream);
    if (st != CHORUS_OK) return st;
  }
  return CHORUS_OK;
}

}  // extern "C"

// ---------------------------------------------------------------------------
// chorus_denoise_run: the whole three-stage request on one stream.
// ---------------------------------------------------------------------------
namespace {

constexpr int kCopyU = 4;  // float4 per thread, all loads issued before the stores

__global__ __launch_bounds__(256) void stream_copy_kernel(float4* __restrict__ dst, const float4* __restrict__ src,
                                                          long n4) {
  const long stride = (long)gridDim.x * blockDim.x;
  const long i0 = (long)blockIdx.x * blockDim.x + threadIdx.x;
  f32x4 v[kCopyU];
#pragma unroll
  for (int u = 0; u < kCopyU; ++u)
    if (i0 + u * stride < n4) v[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(&src[i0 + u * stride]));
#pragma unroll
  for (int u = 0; u < kCopyU; ++u)
    if (i0 + u * stride < n4) __builtin_nontemporal_store(v[u], reinterpret_cast<f32x4*>(&dst[i0 + u * stride]));
}

__global__ void copy_tail_kernel(float* __restrict__ dst, const float* __restrict__ src, long from, long n) {
  long i = from + (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

// g_j = gamma_k where tdiff[j] != 0, else 1  (the per-token key factor of Eq. 2)
__global__ void key_scale_kernel(float* __restrict__ g, const uint8_t* __restrict__ tdiff, int Lt, float gamma_k) {
  int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < Lt) g[j] = (tdiff == nullptr || tdiff[j]) ? gamma_k : 1.0f;
}

int32_t device_copy(float* dst, const float* src, long n, hipStream_t s) {
  if (n <= 0 || dst == src) return CHORUS_OK;
  long n4 = (aligned16(dst) && aligned16(src)) ? n / 4 : 0;
  if (n4 > 0) {
    hipLaunchKernelGGL(stream_copy_kernel, dim3((unsigned)((n4 + 256 * kCopyU - 1) / (256 * kCopyU))), dim3(256), 0, s, (float4*)dst,
                       (const float4*)src, n4);
    CHORUS_LAUNCH_CHECK();
  }
  if (n4 * 4 < n) {
    hipLaunchKernelGGL(copy_tail_kernel, dim3((unsigned)((n - n4 * 4 + 255) / 256)), dim3(256), 0, s, dst, src, n4 * 4,
                       n);
    CHORUS_LAUNCH_CHECK();
  }
  return CHORUS_OK;
}

struct RunWs {
  chorus_lookup_result* lookup;  // device
  int32_t* count;
  int32_t* idx;
  float* key_scale;
  void* lookup_ws;
  size_t lookup_ws_bytes;
  void* compact_ws;
  size_t compact_ws_bytes;
  void* step;
  size_t step_bytes;
  void* text_kv;       // per-block text K / V of this request
  size_t text_kv_bytes;
  void* text_kv_ws;
  size_t text_kv_ws_bytes;
  void* text_kv_uncond;  // the same for the unconditional prompt of classifier-free guidance
  float* x0_prev;        // data predictions of the previous step (multistep solver)
  size_t bytes;
};

RunWs carve_run(const chorus_model_shape& m, int64_t N, void* base) {
  RunWs w;
  const BytePtr p(base);
  size_t off = 0;
  const int64_t Ltok = (int64_t)m.T * (m.Hl / m.ph) * (m.Wl / m.pw);
  auto take = [&](size_t bytes) {
    void* r = p + off;
    off += align_up(bytes, 256);
    return r;
  };
  w.lookup = (chorus_lookup_result*)take(sizeof(chorus_lookup_result));
  w.count = (int32_t*)take(sizeof(int32_t));
  w.idx = (int32_t*)take((size_t)Ltok * 4);
  w.key_scale = (float*)take((size_t)m.block.Lt * 4);
  w.lookup_ws_bytes = chorus_cache_lookup_workspace_bytes(N);
  w.lookup_ws = take(w.lookup_ws_bytes);
  w.compact_ws_bytes = chorus_region_compact_workspace_bytes(Ltok);
  w.compact_ws = take(w.compact_ws_bytes);
  w.step_bytes = chorus_denoise_step_workspace_bytes(&m, Ltok);
  const size_t solver_bytes = chorus_denoise_step_solver_workspace_bytes(&m, Ltok, 1);
  if (solver_bytes > w.step_bytes) w.step_bytes = solver_bytes;
  w.step = take(w.step_bytes);
  w.text_kv_bytes = (size_t)m.n_blocks * chorus_text_kv_bytes(&m.block);
  w.text_kv = take(w.text_kv_bytes);
  w.text_kv_ws_bytes = chorus_text_kv_workspace_bytes(&m.block);
  w.text_kv_ws = take(w.text_kv_ws_bytes);
  w.text_kv_uncond = take(w.text_kv_bytes);
  w.x0_prev = (float*)take((size_t)m.C * m.T * m.Hl * m.Wl * 4);
  w.bytes = off;
  return w;
}

}  // namespace

extern "C" {

size_t chorus_denoise_run_workspace_bytes(const chorus_model_shape* model, int64_t N) {
  if (check_model(model) != CHORUS_OK || N < 0) return 0;
  return carve_run(*model, N, nullptr).bytes;
}

int32_t chorus_stage1_copy(float* latent, const float* SL, int64_t n, void* stream) {
  if (n < 0 || (n > 0 && (!latent || !SL))) return CHORUS_E_ARG;
  return device_copy(latent, SL, (long)n, (hipStream_t)stream);
}

int32_t chorus_cache_insert(float* cache_emb, float* cache_latents, int64_t capacity, int64_t slot, int32_t d,
                            int64_t latent_elems, const float* emb, const float* latent, void* stream) {
  if (!cache_emb || !cache_latents || !emb || !latent) return CHORUS_E_ARG;
  if (capacity <= 0 || slot < 0 || slot >= capacity || d <= 0 || latent_elems <= 0) return CHORUS_E_ARG;
  hipStream_t s = (hipStream_t)stream;
  int32_t st = device_copy(cache_emb + slot * d, emb, d, s);
  if (st != CHORUS_OK) return st;
  return device_copy(cache_latents + slot * latent_elems, latent, (long)latent_elems, s);
}

int32_t chorus_denoise_run(const chorus_model_shape* model, const chorus_block_weights* blocks,
                           const chorus_glue_weights* gw, const chorus_request* rq, float* latent,
                           chorus_run_result* result, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = check_model(model);
  if (st != CHORUS_OK) return st;
  if (!rq || !latent || !result || !gw) return CHORUS_E_ARG;
  if (rq->n_steps < 0 || rq->cache_N < 0 || rq->cache_d <= 0) return CHORUS_E_ARG;
  if (rq->n_steps > 64) return CHORUS_E_SHAPE;
  if (rq->n_steps > 0 && (!rq->sigmas || !rq->t_mods || !rq->t_heads || !rq->text_ctx)) return CHORUS_E_ARG;
  if (!rq->query || (rq->cache_N > 0 && (!rq->cache_emb || !rq->cache_latents))) return CHORUS_E_ARG;
  const int S = rq->latent_steps ? rq->n_latent_steps : 1;  // latents per cache entry
  if (rq->latent_steps) {
    if (S < 1 || S > 64) return CHORUS_E_ARG;
    for (int j = 0; j < S; ++j) {
      if (rq->latent_steps[j] < 1 || rq->latent_steps[j] > rq->n_steps) return CHORUS_E_ARG;
      for (int k = 0; k < j; ++k)
        if (rq->latent_steps[k] == rq->latent_steps[j]) return CHORUS_E_ARG;
    }
    if (rq->store_slot >= rq->cache_N) return CHORUS_E_ARG;
  } else if (rq->store_slot >= 0 &&
             (rq->store_slot >= rq->cache_N || rq->store_after < 1 || rq->store_after > rq->n_steps)) {
    return CHORUS_E_ARG;
  }
  if (rq->solver_order < 0 || rq->solver_order > 2) return CHORUS_E_ARG;
  if (!ws) return CHORUS_E_WORKSPACE;
  const chorus_model_shape& m = *model;
  const bool use_solver = rq->solver_order == 2 || rq->text_ctx_uncond != nullptr;
  RunWs w = carve_run(m, rq->cache_N, ws);
  if (ws_bytes < w.bytes) return CHORUS_E_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const int64_t Ltok = (int64_t)m.T * (m.Hl / m.ph) * (m.Wl / m.pw);
  const int64_t lat_elems = (int64_t)m.C * m.T * m.Hl * m.Wl;
  const int D = m.block.D;

  // stage-1 retrieval, then the scheduler needs the score on the host
  st = chorus_cache_lookup(rq->cache_emb, rq->cache_N, rq->cache_d, rq->query, rq->tau, w.lookup, w.lookup_ws,
                           w.lookup_ws_bytes, stream);
  if (st != CHORUS_OK) return st;
  chorus_lookup_result lr;
  CHORUS_HIP(hipMemcpyAsync(&lr, w.lookup, sizeof(lr), hipMemcpyDeviceToHost, s));
  CHORUS_HIP(hipStreamSynchronize(s));
  result->index = lr.index;
  result->score = lr.score;
  result->hit = lr.hit;

  chorus_step_plan plan_buf[64];
  int32_t K1 = 0, K2 = 0, depth_slot = 0;
  if (rq->latent_steps)
    st = chorus_denoise_schedule_stored(lr.score, rq->tau, rq->n_steps, rq->sched, rq->latent_steps, S, &K1, &K2,
                                        &depth_slot, plan_buf);
  else
    st = chorus_denoise_schedule(lr.score, rq->tau, rq->n_steps, rq->sched, &K1, &K2, plan_buf);
  if (st != CHORUS_OK) return st;
  if (depth_slot < 0) depth_slot = 0;  // no usable depth: the plan has no reuse and SL is never read
  result->K1 = K1;
  result->K2 = K2;
  result->Ls = 0;

  const float* SL = lr.hit ? rq->cache_latents + ((int64_t)lr.index * S + depth_slot) * lat_elems : nullptr;
  int64_t Ls = 0;
  if (K2 > K1) {
    if (!rq->mask_see || !rq->mask_edit) return CHORUS_E_ARG;
    st = chorus_region_compact(rq->mask_see, Ltok, w.idx, w.count, w.compact_ws, w.compact_ws_bytes, stream);
    if (st != CHORUS_OK) return st;
    int32_t cnt = 0;
    CHORUS_HIP(hipMemcpyAsync(&cnt, w.count, sizeof(cnt), hipMemcpyDeviceToHost, s));
    CHORUS_HIP(hipStreamSynchronize(s));
    Ls = cnt;
    result->Ls = cnt;
  }

  // cross-attention keys / values depend only on the prompt: project them once per block for all computed steps
  if (K1 < rq->n_steps && m.n_blocks > 0) {
    st = chorus_model_text_kv_project(model, blocks, rq->text_ctx, w.text_kv, w.text_kv_ws, w.text_kv_ws_bytes, stream);
    if (st != CHORUS_OK) return st;
    if (rq->text_ctx_uncond) {
      st = chorus_model_text_kv_project(model, blocks, rq->text_ctx_uncond, w.text_kv_uncond, w.text_kv_ws,
                                        w.text_kv_ws_bytes, stream);
      if (st != CHORUS_OK) return st;
    }
  }

  // which tokens hold a data prediction from the previous step: 0 none, 1 the M_see tokens, 2 all
  int history = 0;
  for (int i = 0; i < rq->n_steps; ++i) {
    const chorus_step_plan& p = plan_buf[i];
    if (p.stage == 1) {
      // full reuse: only the last reused step's latent survives
      if (i == K1 - 1) {
        st = device_copy(latent, SL, (long)lat_elems, s);
        if (st != CHORUS_OK) return st;
      }
      continue;
    }
    const float* ks = nullptr;
    if (p.gamma_k != 1.0f) {
      hipLaunchKernelGGL(key_scale_kernel, dim3((unsigned)((m.block.Lt + 255) / 256)), dim3(256), 0, s, w.key_scale,
                         rq->tdiff, m.block.Lt, p.gamma_k);
      CHORUS_LAUNCH_CHECK();
      ks = w.key_scale;
    }
    const float dsigma = rq->sigmas[i + 1] - rq->sigmas[i];
    const float* t_mod = rq->t_mods + (size_t)i * 6 * D;
    const float* t_head = rq->t_heads + (size_t)i * 2 * D;
    if (use_solver) {
      chorus_sampler_coef cf;
      st = chorus_sampler_coefficients(rq->sigmas, rq->n_steps, i, (history && rq->solver_order == 2) ? 2 : 1, &cf);
      if (st != CHORUS_OK) return st;
      const void* kv = m.n_blocks > 0 ? w.text_kv : nullptr;
      const void* kvu = (m.n_blocks > 0 && rq->text_ctx_uncond) ? w.text_kv_uncond : nullptr;
      const uint8_t* hist = history == 1 ? rq->mask_see : nullptr;
      if (p.stage == 2) {
        // the latent outside M_see already is the source latent once a reused step or an earlier stage-2 step ran
        st = chorus_denoise_step_solver(model, blocks, gw, latent, w.idx, Ls, kv, kvu, rq->guidance, t_mod, t_head, ks,
                                        p.gamma_o, &cf, w.x0_prev, hist, SL, rq->mask_edit, i > 0, w.step, w.step_bytes,
                                        stream);
        history = 1;
      } else {
        st = chorus_denoise_step_solver(model, blocks, gw, latent, nullptr, Ltok, kv, kvu, rq->guidance, t_mod, t_head,
                                        ks, p.gamma_o, &cf, w.x0_prev, hist, nullptr, nullptr, 0, w.step, w.step_bytes,
                                        stream);
        history = 2;
      }
    } else if (p.stage == 2) {
      // as above: after a reused step or an earlier stage-2 step Eq. 6 only has to touch the selected tokens
      st = denoise_step_impl(model, blocks, gw, latent, w.idx, Ls, rq->text_ctx, m.n_blocks > 0 ? (const uint8_t*)w.text_kv : nullptr,
                             t_mod, t_head, ks, p.gamma_o, dsigma, SL, rq->mask_edit, i > 0, w.step, w.step_bytes, stream);
    } else {
      st = denoise_step_impl(model, blocks, gw, latent, nullptr, Ltok, rq->text_ctx, m.n_blocks > 0 ? (const uint8_t*)w.text_kv : nullptr,
                             t_mod, t_head, ks, p.gamma_o, dsigma, nullptr, nullptr, false, w.step, w.step_bytes, stream);
    }
    if (st != CHORUS_OK) return st;
    // cache update after a miss: keep the prompt embedding and this intermediate latent for later requests
    if (!lr.hit && rq->store_slot >= 0 && !rq->latent_steps && i + 1 == rq->store_after) {
      st = chorus_cache_insert(rq->cache_emb, rq->cache_latents, rq->cache_N, rq->store_slot, rq->cache_d, lat_elems,
                               rq->query, latent, stream);
      if (st != CHORUS_OK) return st;
    }
    if (!lr.hit && rq->store_slot >= 0 && rq->latent_steps) {
      // the prompt embedding goes in with the shallowest stored state: no key without a latent, and one copy of it
      int shallowest = rq->latent_steps[0];
      for (int j = 1; j < S; ++j) shallowest = rq->latent_steps[j] < shallowest ? rq->latent_steps[j] : shallowest;
      for (int j = 0; j < S; ++j) {
        if (rq->latent_steps[j] != i + 1) continue;
        st = device_copy(rq->cache_latents + ((int64_t)rq->store_slot * S + j) * lat_elems, latent, (long)lat_elems, s);
        if (st != CHORUS_OK) return st;
      }
      if (i + 1 == shallowest) {
        st = device_copy(rq->cache_emb + rq->store_slot * (int64_t)rq->cache_d, rq->query, rq->cache_d, s);
        if (st != CHORUS_OK) return st;
      }
    }
  }
  return CHORUS_OK;
}

}  // extern "C"
