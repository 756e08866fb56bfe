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
  uint8_t* p = (uint8_t*)base;
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

int32_t chorus_denoise_step(const chorus_model_shape* model, const chorus_block_weights* blocks,
                            const chorus_glue_weights* gw, float* latent, const int32_t* token_idx, int64_t Ls,
                            const uint16_t* text_ctx, const float* t_mod, const float* t_head,
                            const float* tgaa_key_scale, float gamma_o, float dsigma, const float* SL,
                            const uint8_t* mask_edit, void* ws, size_t ws_bytes, void* stream) {
  int32_t st = check_model(model);
  if (st != CHORUS_OK) return st;
  const chorus_model_shape& m = *model;
  const int64_t Ltok = (int64_t)m.T * (m.Hl / m.ph) * (m.Wl / m.pw);
  if (Ls < 0 || Ls > Ltok) return CHORUS_E_ARG;
  if (!token_idx && Ls != Ltok) return CHORUS_E_ARG;
  if (!latent || !gw || !text_ctx || !t_mod || !t_head || (m.n_blocks > 0 && !blocks)) return CHORUS_E_ARG;
  if ((mask_edit != nullptr) != (SL != nullptr)) return CHORUS_E_ARG;
  if (!ws) return CHORUS_E_WORKSPACE;
  StepWs w = carve_step(m, Ls, ws);
  if (ws_bytes < w.bytes) return CHORUS_E_WORKSPACE;
  if (Ls > 0) {
    st = chorus_patch_embed(latent, m.C, m.T, m.Hl, m.Wl, m.ph, m.pw, token_idx, Ls, gw, m.block.D, w.x, w.glue,
                            w.glue_bytes, stream);
    if (st != CHORUS_OK) return st;
    for (int b = 0; b < m.n_blocks; ++b) {
      st = chorus_dit_block_step(&m.block, &blocks[b], w.x, Ls, token_idx, text_ctx, t_mod, tgaa_key_scale, gamma_o,
                                 w.block, w.block_bytes, stream);
      if (st != CHORUS_OK) return st;
    }
    st = chorus_head_update(latent, w.x, Ls, token_idx, gw, t_head, dsigma, m.block.D, m.C, m.T, m.Hl, m.Wl, m.ph,
                            m.pw, w.glue, w.glue_bytes, stream);
    if (st != CHORUS_OK) return st;
  }
  if (mask_edit) {
    st = chorus_region_blend(latent, latent, SL, mask_edit, m.C, m.T, m.Hl, m.Wl, m.ph, m.pw, stream);
    if (st != CHORUS_OK) return st;
  }
  return CHORUS_OK;
}

}  // extern "C"
