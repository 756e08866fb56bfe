/*
 * chorus_ops.h -- the individual device operations chorus_dit_block_step is made
 * of, plus the step glue around the block stack. Exported so that each kernel can
 * be checked against the CPU oracle and timed on its own. Same conventions as
 * chorus.h (status codes, dev pointers, stream, bf16 as uint16_t).
 */
#ifndef CHORUS_OPS_H
#define CHORUS_OPS_H

#include <math.h>

#include "chorus.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------------
 * C = epilogue(A W^T + bias): the QKV / O / FFN projections of the block
 * (Sec. 2.1; the FLOPs next to attention). bf16 operands, fp32 accumulate on MFMA.
 *   A    dev [M, K] bf16 row-major (lda = K)
 *   W    dev [N, K] bf16 row-major (a weight matrix as stored: [out, in])
 *   bias dev [N] fp32 or NULL
 *   epilogue  CHORUS_EPI_*:
 *     BF16       out bf16 [M,N] = acc + bias
 *     GELU_BF16  out bf16 [M,N] = gelu_tanh(acc + bias)
 *     F32        out fp32 [M,N] = acc + bias
 *     RESID      out fp32 [M,N] += (gate0[n] + gate1[n]) * scale * (acc + bias)
 *                (gate0/gate1 dev [N] fp32, either may be NULL = 0; both NULL = 1):
 *                the gated residual of the AdaLN block and, with scale = gamma_o and
 *                no gates, the TGAA output amplification of Eq. 3
 * K % 64 == 0, N % 8 == 0, M >= 0 arbitrary.
 * ------------------------------------------------------------------------ */
#define CHORUS_EPI_BF16 0
#define CHORUS_EPI_GELU_BF16 1
#define CHORUS_EPI_F32 2
#define CHORUS_EPI_RESID 3
int32_t chorus_gemm_bf16(const uint16_t* A, const uint16_t* W, int64_t M, int32_t N, int32_t K, int32_t epilogue,
                         void* out, const float* bias, const float* gate0, const float* gate1, float scale,
                         void* stream);

/* chorus_gemm_bf16 with the tile kernel named by the caller, for tests and comparisons (every kernel is correct on
 * every shape the call accepts; only the speed differs): kernel 0 = the default choice by problem size,
 * 1 = 128 x 64 register-staged tiles, 2 = 256 x 128 register-staged tiles, 3 = 256 x 256 direct-to-LDS tiles,
 * 4 = 128 x 128 direct-to-LDS tiles. Anything else: CHORUS_E_ARG. */
int32_t chorus_gemm_bf16_kernel(const uint16_t* A, const uint16_t* W, int64_t M, int32_t N, int32_t K, int32_t epilogue,
                                void* out, const float* bias, const float* gate0, const float* gate1, float scale,
                                int32_t kernel, void* stream);

/* out bf16 [L, D] = LN(x) * (mul_base + mul0 + mul1) + (add0 + add1), LN over D without
 * affine, eps 1e-6; mul_base = 1 if plus_one else 0; mul1/add1 may be NULL.
 * AdaLN modulation: mul = scale rows of (table, t_mod), add = shift rows, plus_one = 1.
 * Affine LayerNorm: mul0 = weight, add0 = bias, plus_one = 0.  x dev [L, D] fp32.
 * D a multiple of 4, at most 8192 (CHORUS_E_SHAPE otherwise). */
int32_t chorus_ln_modulate(const float* x, uint16_t* out, int64_t L, int32_t D, const float* mul0, const float* mul1,
                           const float* add0, const float* add1, int32_t plus_one, void* stream);

/* RMSNorm over the full width D = H*dh with a learned gain, then (rope != 0) 3-D
 * RoPE at the token's original grid position, written head-major:
 *   in  dev bf16, row i at in + i*ld, D values
 *   out dev bf16 [H, Lpad, dh]; rows L..Lpad-1 are written as zeros
 *   token_idx dev [L] int32 or NULL (identity)
 *   out_scale: finite, > 0; every output is multiplied by it in fp32 before the one rounding to bf16 (1 for the
 *   plain operation; the block passes CHORUS_ATTENTION_Q_PRESCALE(dh) for the queries of chorus_attention's
 *   variant 6). CHORUS_E_ARG otherwise. */
int32_t chorus_qk_norm_rope(const uint16_t* in, int64_t ld, const float* gain, uint16_t* out, int64_t L, int64_t Lpad,
                            int32_t H, int32_t dh, const int32_t* token_idx, int32_t gT, int32_t gH, int32_t gW,
                            int32_t rope, float out_scale, void* stream);

/* V [L, D] (row i at in + i*ld) -> Vt [D, Lpad], zero beyond L, with the token order
 * inside every group of 16 permuted to the attention kernel's operand order:
 * position 8c + 4u + i of a group holds token 8u + 4c + i (c, u in {0,1}, i < 4).
 * D % 64 == 0, Lpad % 64 == 0. */
int32_t chorus_v_transpose(const uint16_t* in, int64_t ld, uint16_t* out, int64_t L, int64_t Lpad, int32_t D,
                           void* stream);

/* O = softmax(col_scale_j * (Q K^T)/sqrt(dh)) V per head (flash-style, online softmax,
 * never materialises the logits). Self-attention of the block with col_scale NULL;
 * cross-attention with TGAA key amplification (Eq. 2) with col_scale = the per-text-
 * token factor (scaling a key scales its logit column).
 *   Q   dev bf16 [H, LqPad, dh]     K dev bf16 [H, LkPad, dh]
 *   Vt  dev bf16 [H*dh, LkPad] in chorus_v_transpose's layout
 *   O   dev bf16 [Lq, H*dh] token-major
 *   col_scale dev [Lk] fp32, 16-byte aligned, or NULL
 * dh in {64,128}; LkPad % 64 == 0, LkPad >= Lk >= 1; rows/cols beyond Lq/Lk are padding
 * (finite values).
 * variant: 0 = the default choice (128-key tiles on 16x16x32 MFMAs when
 * CHORUS_ATTENTION_LONG_KEYS(Lk, LkPad): LkPad % 128 == 0 and Lk >= 512; else 64-key tiles on 32x32x16 MFMAs);
 * 3 = 64-key tiles; 5 = 128-key tiles on
 * 16x16x32 MFMAs; 6 = as 5 for a Q that holds the queries already multiplied by log2(e) / sqrt(dh)
 * (CHORUS_ATTENTION_Q_PRESCALE(dh), applied in fp32 by the producer before its rounding to bf16): the same
 * function of the unscaled queries, with one vector instruction less per logit when col_scale is NULL. 5 and 6
 * give CHORUS_E_SHAPE when LkPad % 128 != 0. Any other value: CHORUS_E_ARG. */
#define CHORUS_ATTENTION_Q_PRESCALE(dh) (1.4426950408889634f / sqrtf((float)(dh)))
#define CHORUS_ATTENTION_LONG_KEYS(Lk, LkPad) ((LkPad) % 128 == 0 && (Lk) >= 512)
int32_t chorus_attention(const uint16_t* Q, const uint16_t* K, const uint16_t* Vt, uint16_t* O,
                         const float* col_scale, int64_t Lq, int64_t Lk, int64_t LqPad, int64_t LkPad, int32_t H,
                         int32_t dh, int32_t variant, void* stream);

/* ------------------------------------------------------------------------
 * Step glue (stand-ins that close the denoising loop around the blocks; the
 * paper's sampler is DPM++ with default settings, whose coefficients it does not
 * give, so an Euler update x <- x + dsigma * v is used).
 * patch_embed: x[i, :] = patch(latent, token_idx[i]) Wp^T + bp for the Ls selected
 *   tokens; a patch is the (c, dy, dx) values of a 1 x ph x pw cell.
 * head_update: v = (LN(x)(1 + scale) + shift) Wh^T + bh with (shift, scale) =
 *   head_table + t_head; latent[patch of token_idx[i]] += dsigma * v[i].
 * text_project: ctx = gelu_tanh(text W1^T + b1) W2^T + b2 -> bf16 [Lt, D].
 * ------------------------------------------------------------------------ */
typedef struct {
  const uint16_t* w_patch; /* [D, P] bf16, P = C*ph*pw (multiple of 64) */
  const float* b_patch;    /* [D] */
  const uint16_t* w_head;  /* [P, D] bf16 */
  const float* b_head;     /* [P] */
  const float* head_table; /* [2, D]: shift, scale */
} chorus_glue_weights;

size_t chorus_glue_workspace_bytes(int32_t D, int32_t P, int64_t Ls);
int32_t chorus_patch_embed(const float* latent, int32_t C, int32_t T, int32_t Hl, int32_t Wl, int32_t ph, int32_t pw,
                           const int32_t* token_idx, int64_t Ls, const chorus_glue_weights* gw, int32_t D, float* x,
                           void* ws, size_t ws_bytes, void* stream);
int32_t chorus_head_update(float* latent, const float* x, int64_t Ls, const int32_t* token_idx,
                           const chorus_glue_weights* gw, const float* t_head, float dsigma, int32_t D, int32_t C,
                           int32_t T, int32_t Hl, int32_t Wl, int32_t ph, int32_t pw, void* ws, size_t ws_bytes,
                           void* stream);
/* chorus_head_update with Eq. 6 applied to the selected tokens in the same pass: a selected token n with
 * mask_edit[n] == 0 receives SL (device fp32, the latent's shape) instead of the update. With SL and mask_edit NULL it
 * is chorus_head_update. A caller whose latent already equals SL outside the selection (after a stage-1 copy or an
 * earlier region step) needs no separate chorus_region_blend then. latent and SL must not overlap.
 * CHORUS_E_ARG when only one of SL / mask_edit is given; otherwise as chorus_head_update. */
int32_t chorus_head_update_region(float* latent, const float* x, int64_t Ls, const int32_t* token_idx,
                                  const chorus_glue_weights* gw, const float* t_head, float dsigma, const float* SL,
                                  const uint8_t* mask_edit, int32_t D, int32_t C, int32_t T, int32_t Hl, int32_t Wl,
                                  int32_t ph, int32_t pw, void* ws, size_t ws_bytes, void* stream);
/* ------------------------------------------------------------------------
 * The sampler (Sec. 4.1: the DPM++ solver with default settings; the paper gives no
 * formulas): DPM-Solver++ in data-prediction form, multistep, order <= 2, on the
 * rectified-flow path x_sigma = alpha x0 + sigma eps, alpha = 1 - sigma, whose velocity
 * v = eps - x0 the model predicts. With lambda = log(alpha / sigma), h = lambda_t - lambda_s,
 * r = h_prev / h, one step from sigma_s to sigma_t is
 *     x0 = x_s - sigma_s v
 *     D  = x0                                   (first order, or no history)
 *        = (1 + 1/(2r)) x0 - (1/(2r)) x0_prev   (second order)
 *     x_t = (sigma_t / sigma_s) x_s - alpha_t (exp(-h) - 1) D
 * chorus_head_update (above) is the first-order step in its Euler form x_s + (sigma_t - sigma_s) v.
 *
 * chorus_sampler_coefficients (host-only): the weights of step i of a schedule.
 *   sigmas host [n_steps + 1], strictly decreasing, sigmas[0] <= 1, sigmas[n_steps] >= 0
 *   order 1 or 2. Step 0 (no earlier level), a step that ends at sigma = 0 (h is infinite)
 *   and a previous level of exactly 1 (lambda = -inf) give first-order weights.
 *   Errors: CHORUS_E_ARG (null pointer, i outside [0, n_steps), order, levels out of order).
 *
 * chorus_head_update_solver: head + sampler step on the selected tokens in one pass over them:
 *   v = head(x), or head(x_uncond) + guidance (head(x) - head(x_uncond)) when x_uncond is
 *   given (classifier-free guidance; x, x_uncond dev [Ls, D] fp32);
 *   x0_prev dev [C, T, Hl, Wl] fp32: read where the second-order form applies, then
 *     overwritten with this step's x0 on every selected token (NULL: keep no history;
 *     needs coef->c1 == 0);
 *   hist dev [T*Hg*Wg] uint8 or NULL: tokens whose x0_prev entry is valid (NULL = all);
 *     the others take the first-order form;
 *   SL, mask_edit (both or neither): Eq. 6 on the selected tokens -- a selected token
 *     with mask_edit = 0 receives SL instead of the update. Tokens that are not selected
 *     are not touched.
 *   latent, x0_prev and SL must not overlap. Workspace: chorus_head_solver_workspace_bytes.
 * ------------------------------------------------------------------------ */
typedef struct {
  float sigma_s; /* noise level of the step's input */
  float rho;     /* sigma_t / sigma_s */
  float A;       /* -alpha_t (exp(-h) - 1) = alpha_t - sigma_t alpha_s / sigma_s */
  float c0, c1;  /* D = c0 x0 + c1 x0_prev on tokens with history; (1, 0): first order */
} chorus_sampler_coef;

int32_t chorus_sampler_coefficients(const float* sigmas, int32_t n_steps, int32_t i, int32_t order,
                                    chorus_sampler_coef* out);
size_t chorus_head_solver_workspace_bytes(int32_t D, int32_t P, int64_t Ls, int32_t cfg);
int32_t chorus_head_update_solver(float* latent, const float* x, const float* x_uncond, float guidance, int64_t Ls,
                                  const int32_t* token_idx, const chorus_glue_weights* gw, const float* t_head,
                                  const chorus_sampler_coef* coef, float* x0_prev, const uint8_t* hist, const float* SL,
                                  const uint8_t* mask_edit, int32_t D, int32_t C, int32_t T, int32_t Hl, int32_t Wl,
                                  int32_t ph, int32_t pw, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Timestep injection (Sec. 2.1, Fig. 2): the projected timestep embedding of one step, i.e.
 * the t_mod [6, D] and t_head [2, D] inputs of the block, step and run calls.
 *   f = [cos(t w_i), sin(t w_i)], w_i = 10000^(-i / half), half = freq_dim / 2
 *   e = W2 silu(W1 f + b1) + b2;  t_mod = reshape(Wp silu(e) + bp, [6, D]);  t_head = [e, e]
 *   weights: bf16 [out, in] (w_t1 [D, freq_dim], w_t2 [D, D], w_tp [6 D, D]), fp32 biases (NULL = 0)
 *   t_mod, t_head dev fp32 (written); ws: chorus_time_mod_workspace_bytes(D, freq_dim)
 * freq_dim and D multiples of 8. For a fixed schedule the results are per-model constants:
 * compute them once per noise level and keep them.
 * ------------------------------------------------------------------------ */
typedef struct {
  const uint16_t* w_t1;
  const float* b_t1;
  const uint16_t* w_t2;
  const float* b_t2;
  const uint16_t* w_tp;
  const float* b_tp;
} chorus_time_weights;

size_t chorus_time_mod_workspace_bytes(int32_t D, int32_t freq_dim);
int32_t chorus_time_mod(float t, int32_t freq_dim, int32_t D, const chorus_time_weights* w, float* t_mod, float* t_head,
                        void* ws, size_t ws_bytes, void* stream);

size_t chorus_text_project_workspace_bytes(int32_t Lt, int32_t D);
int32_t chorus_text_project(const uint16_t* text, int32_t Lt, int32_t text_dim, int32_t D, const uint16_t* w1,
                            const float* b1, const uint16_t* w2, const float* b2, uint16_t* ctx, void* ws,
                            size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * One computed denoising step (Sec. 3.1: a stage-2 or stage-3 step) in one call:
 *   x = patch_embed(latent[token_idx]); x = block_b(x) for every block;
 *   latent[token_idx] += dsigma * head(x); then, when mask_edit is given (stage 2),
 *   latent = M_edit ? latent : SL (Eq. 6).
 * Stage 2 passes the compacted list of the visible mask M_see as token_idx (from
 * chorus_region_compact) and the edit mask M_edit for the fusion; all M_see tokens
 * go through every layer, only M_edit tokens survive the fusion (Sec. 3.3.2).
 * Stage 3 passes token_idx = NULL, Ls = all tokens, SL = mask_edit = NULL.
 *   blocks host array [n_blocks] of structs of device pointers
 *   latent dev [C, T, Hl, Wl] fp32 in/out;  SL same shape
 *   t_mod dev [6, D], t_head dev [2, D] fp32: projected timestep embedding of this step
 *   tgaa_key_scale dev [Lt] fp32, 16-byte aligned, or NULL; gamma_o: as in chorus_dit_block_step
 * The patch is 1 x ph x pw; the block's token grid must be (T, Hl/ph, Wl/pw).
 * ------------------------------------------------------------------------ */
typedef struct {
  chorus_block_shape block;
  int32_t C, T, Hl, Wl, ph, pw;
  int32_t n_blocks;
} chorus_model_shape;

size_t chorus_denoise_step_workspace_bytes(const chorus_model_shape* model, int64_t Ls);
int32_t chorus_denoise_step(const chorus_model_shape* model, const chorus_block_weights* blocks,
                            const chorus_glue_weights* gw, float* latent, const int32_t* token_idx, int64_t Ls,
                            const uint16_t* text_ctx, const float* t_mod, const float* t_head,
                            const float* tgaa_key_scale, float gamma_o, float dsigma, const float* SL,
                            const uint8_t* mask_edit, void* ws, size_t ws_bytes, void* stream);
/* The same step with the prompt given as the per-block text keys / values that
 * chorus_model_text_kv_project makes once per request (block b's entry at
 * text_kv + b * chorus_text_kv_bytes(&model->block)); results are bit-identical to
 * chorus_denoise_step. chorus_model_text_kv_project needs a workspace of
 * chorus_text_kv_workspace_bytes(&model->block). */
size_t chorus_model_text_kv_bytes(const chorus_model_shape* model);
int32_t chorus_model_text_kv_project(const chorus_model_shape* model, const chorus_block_weights* blocks,
                                     const uint16_t* text_ctx, void* text_kv, void* ws, size_t ws_bytes, void* stream);
int32_t chorus_denoise_step_kv(const chorus_model_shape* model, const chorus_block_weights* blocks,
                               const chorus_glue_weights* gw, float* latent, const int32_t* token_idx, int64_t Ls,
                               const void* text_kv, const float* t_mod, const float* t_head,
                               const float* tgaa_key_scale, float gamma_o, float dsigma, const float* SL,
                               const uint8_t* mask_edit, void* ws, size_t ws_bytes, void* stream);

/* One computed step with the multistep solver and, optionally, classifier-free guidance:
 *   x = patch_embed(latent[token_idx]); x_c = blocks(x; text_kv, TGAA);
 *   x_u = blocks(x; text_kv_uncond, no TGAA) when text_kv_uncond is given;
 *   chorus_head_update_solver(latent, x_c, x_u, ...) with Eq. 6 folded into its pass.
 * TGAA (key scale, gamma_o) belongs to the conditional branch only: an unconditional
 * prompt has no differential tokens.
 *   text_kv, text_kv_uncond: from chorus_model_text_kv_project
 *   coef: chorus_sampler_coefficients of this step (host struct, copied at the call)
 *   x0_prev, hist: as in chorus_head_update_solver
 *   SL, mask_edit (both or neither): stage 2. Eq. 6 also resets the tokens outside
 *     token_idx to SL; outside_is_source != 0 states that they already hold SL (true after
 *     the stage-1 copy and after any earlier stage-2 step with the same SL), and then no
 *     extra pass over the latent is made; with 0, chorus_region_blend runs afterwards.
 * Workspace: chorus_denoise_step_solver_workspace_bytes(model, Ls, cfg) with cfg != 0 iff
 * text_kv_uncond is given. Errors as chorus_denoise_step. */
size_t chorus_denoise_step_solver_workspace_bytes(const chorus_model_shape* model, int64_t Ls, int32_t cfg);
int32_t chorus_denoise_step_solver(const chorus_model_shape* model, const chorus_block_weights* blocks,
                                   const chorus_glue_weights* gw, float* latent, const int32_t* token_idx, int64_t Ls,
                                   const void* text_kv, const void* text_kv_uncond, float guidance, const float* t_mod,
                                   const float* t_head, const float* tgaa_key_scale, float gamma_o,
                                   const chorus_sampler_coef* coef, float* x0_prev, const uint8_t* hist, const float* SL,
                                   const uint8_t* mask_edit, int32_t outside_is_source, void* ws, size_t ws_bytes,
                                   void* stream);

/* ------------------------------------------------------------------------
 * The whole three-stage request (Sec. 3.1) on one stream:
 *   1. top-1 cosine lookup of `query` in the cache; the score m is read back
 *   2. (K1, K2) and the per-step TGAA factors from chorus_denoise_schedule
 *   3. steps [0, K1): full reuse -- the matched entry's cached latent replaces `latent`
 *      steps [K1, K2): compact M_see once, then chorus_denoise_step on those tokens with
 *        key scale g_j = gamma_k on the differential tokens (tdiff[j] != 0; tdiff NULL
 *        = every token), output amplification gamma_o, and fusion with the cached
 *        latent under M_edit (Eq. 6)
 *      steps [K2, N): chorus_denoise_step on all tokens
 *      (the text keys / values of every block are projected once, before the first computed step)
 * A miss (m < tau, or an empty cache) runs N plain steps from the caller's latent.
 * Cache update: when store_slot >= 0 and the request is a miss, the query and the latent after
 * store_after steps (1 <= store_after <= n_steps; the intermediate state a later hit with
 * K1 = store_after resumes from) are written to entry store_slot with chorus_cache_insert.
 * One cached latent per entry serves both the stage-1 copy and the stage-2 fusion. With latent_steps NULL the
 * library does not know at which depth that latent was taken and resumes from it at whatever K1 Eq. 1 gives:
 * correct only when the caller's entries were stored at that K1 (a fixed N and a plan whose K1 does not move
 * with the score, as in the benchmark's 4-step configuration). A caller that knows the depth passes it as
 * latent_steps = {depth}, n_latent_steps = 1 (the same memory layout): K1 is then snapped to it, and a score
 * whose K1 falls below it runs as a miss instead of resuming from a latent at the wrong noise level.
 * Several depths per entry: with latent_steps (host [n_latent_steps], distinct, each in [1, n_steps])
 * cache_latents is [N, n_latent_steps, C, T, Hl, Wl]; a hit takes its boundaries from
 * chorus_denoise_schedule_stored and resumes from the latent stored at depth K1 (also the SL of the
 * stage-2 fusion); a miss with store_slot >= 0 writes the latent after latent_steps[j] steps to
 * [store_slot, j] for every j and the query once (store_after is then ignored).
 * Sampler: solver_order 0 or 1 with text_ctx_uncond NULL takes the Euler form of the first-order
 * step (chorus_denoise_step); solver_order 2 and / or text_ctx_uncond (classifier-free guidance
 * with scale `guidance`, two model evaluations per step) take chorus_denoise_step_solver. The
 * history of data predictions starts empty at the first computed step; a token that a step did
 * not compute (outside M_see in stage 2) has none in the next, so the first stage-3 step after
 * stage 2 is second-order on the M_see tokens and first-order elsewhere.
 * Two host synchronisations: after the lookup and after the compaction count.
 *   cache_emb dev [N, d]; cache_latents dev [N, C, T, Hl, Wl] fp32; query dev [d]
 *   sigmas host [n_steps + 1]; t_mods dev [n_steps, 6, D]; t_heads dev [n_steps, 2, D]
 *   text_ctx dev [Lt, D] bf16; tdiff dev [Lt] uint8 or NULL
 *   mask_see, mask_edit dev [T*Hg*Wg] uint8 (needed only if a stage-2 step is planned)
 *   sched: NULL = default schedule parameters;  n_steps <= 64
 *   latent dev [C, T, Hl, Wl] fp32: initial noise in, final latent out
 *   result host
 * chorus_stage1_copy is the full-reuse copy on its own (n fp32 elements).
 * ------------------------------------------------------------------------ */
typedef struct {
  float* cache_emb;      /* read; entry store_slot is written on a miss */
  float* cache_latents;
  int64_t cache_N;
  int32_t cache_d;
  const float* query;
  float tau;
  const chorus_sched_params* sched;
  int32_t n_steps;
  const float* sigmas;
  const float* t_mods;
  const float* t_heads;
  const uint16_t* text_ctx;
  const uint8_t* tdiff;
  const uint8_t* mask_see;
  const uint8_t* mask_edit;
  int64_t store_slot;    /* -1: no cache update */
  int32_t store_after;
  const int32_t* latent_steps;      /* host; NULL: one latent per entry, used whatever K1 is */
  int32_t n_latent_steps;
  int32_t solver_order;             /* 0, 1: first order; 2: DPM-Solver++ multistep */
  const uint16_t* text_ctx_uncond;  /* dev [Lt, D] bf16 or NULL: classifier-free guidance */
  float guidance;
} chorus_request;

typedef struct {
  int32_t index;
  float score;
  int32_t hit;
  int32_t K1, K2;
  int32_t Ls; /* tokens computed in a stage-2 step (0 if none was planned) */
} chorus_run_result;

size_t chorus_denoise_run_workspace_bytes(const chorus_model_shape* model, int64_t N);
int32_t chorus_denoise_run(const chorus_model_shape* model, const chorus_block_weights* blocks,
                           const chorus_glue_weights* gw, const chorus_request* rq, float* latent,
                           chorus_run_result* result, void* ws, size_t ws_bytes, void* stream);
int32_t chorus_stage1_copy(float* latent, const float* SL, int64_t n, void* stream);

/* ------------------------------------------------------------------------
 * Region masks (Sec. 3.3.1 "Region Mask Generation" stages 2-3; Sec. 3.3.2, Eq. 5).
 * Byte masks on the device, any non-zero byte is "set"; outputs hold 0 / 1. Exact.
 *
 * chorus_mask_pooled_extent (host-only): number of windows along an axis of n sites cut
 * into windows of k after `lead` leading sites that are windows of their own
 * (lead + ceil((n - lead) / k)); CHORUS_E_ARG (negative) for k < 1, lead < 0 or lead > n.
 *
 * chorus_mask_project: key-frame propagation fused with the max-pool projection from
 * pixel space to the latent / token grid.
 *   key_masks  dev [Kf, Hp, Wp] uint8, the segmentation masks of the key frames
 *   frame_key  dev [Tp] int32, key frame of every frame's temporal group; NULL = every
 *              frame is its own key frame (then Kf must equal Tp). An entry outside
 *              [0, Kf) makes that frame contribute nothing.
 *   window     (kt, kh, kw), stride = window, windows are cut at the far edge; along time
 *              the first t_lead frames map to one output frame each (a causal video VAE
 *              encodes the first frame alone: 81 frames, kt = 4, t_lead = 1 -> 21)
 *   out        dev [To, Ho, Wo] uint8 with the extents chorus_mask_pooled_extent gives;
 *              out[t,y,x] = 1 iff any site of the window is set. Must not overlap key_masks.
 * Wp up to 65536. Errors: CHORUS_E_ARG (null pointer, window < 1, t_lead outside [0, Tp],
 * frame_key NULL with Kf != Tp), CHORUS_E_SHAPE (extent limits), CHORUS_E_HIP.
 *
 * chorus_mask_hierarchy: Eq. 5, M_edit = I(M_base * K_r > 0), M_see = I(M_base * K_r' > 0)
 * with all-ones box kernels of 2 r + 1 sites per axis; sites beyond the grid count as 0.
 *   mask_base  dev [T, H, W] uint8
 *   r_edit, r_see  host int32[3] = radii along (t, h, w); r_see[a] >= r_edit[a] >= 0,
 *              which gives M_see >= M_edit >= M_base. r_edit may be NULL iff mask_edit is.
 *   mask_edit, mask_see  dev [T, H, W] uint8; either may be NULL (not both); neither may
 *              overlap mask_base.
 * Errors: CHORUS_E_ARG, CHORUS_E_SHAPE (more than 2^31 - 257 sites), CHORUS_E_HIP.
 * Both calls are asynchronous on `stream` and allocate nothing.
 * ---------------------------------------------------------------------- */
int32_t chorus_mask_pooled_extent(int32_t n, int32_t k, int32_t lead);
int32_t chorus_mask_project(const uint8_t* key_masks, int32_t Kf, const int32_t* frame_key, int32_t Tp, int32_t Hp,
                            int32_t Wp, int32_t kt, int32_t kh, int32_t kw, int32_t t_lead, uint8_t* out, void* stream);
int32_t chorus_mask_hierarchy(const uint8_t* mask_base, int32_t T, int32_t H, int32_t W, const int32_t r_edit[3],
                              const int32_t r_see[3], uint8_t* mask_edit, uint8_t* mask_see, void* stream);

/* ------------------------------------------------------------------------
 * Per-kernel timing for benchmarks. chorus_prof_enable takes a bit mask of kernel
 * classes (bit c = class c; 0 = off, the default). For the enabled classes
 * chorus_dit_block_step brackets the launches with HIP events on the caller's
 * stream; chorus_prof_read waits for them and returns the summed milliseconds and
 * the launch count of one class since the last reset. Not thread-safe.
 * ------------------------------------------------------------------------ */
#define CHORUS_PROF_SELF_ATTN 0
#define CHORUS_PROF_CROSS_ATTN 1
#define CHORUS_PROF_GEMM 2
#define CHORUS_PROF_NORM 3
#define CHORUS_PROF_CLASSES 4
int32_t chorus_prof_enable(int32_t class_mask);
int32_t chorus_prof_reset(void);
int32_t chorus_prof_read(int32_t kernel_class, double* total_ms, int32_t* launches);

/* ------------------------------------------------------------------------
 * Measured matrix-pipe ceiling, for benchmarks. Runs a loop of bf16 16x16x32 MFMAs on every
 * CU (two waves per SIMD, each result block accumulated by four MFMAs in a row, the order of the
 * self-attention kernel), `launches` launches after a warm-up of twice as many, and returns the
 * sustained TFLOP/s. The part is power-managed, so the result depends on the operand values and
 * on what accompanies the MFMAs:
 *   normal_data  0: every operand element is 1.0;  1: N(0,1) values (a fixed hash)
 *   mix          bit 0: the A operand of every pair of MFMAs is read from LDS (1 KB per pair, what
 *                       a kernel with 32 result rows per wave needs);
 *                bit 1: one exp2 and one maximum per pair of MFMAs (per logit of the softmax)
 *   ws           dev, chorus_mfma_ceiling_workspace_bytes() bytes (results are discarded)
 * Synchronises the stream. Errors: CHORUS_E_ARG, CHORUS_E_WORKSPACE, CHORUS_E_HIP.
 * ------------------------------------------------------------------------ */
size_t chorus_mfma_ceiling_workspace_bytes(void);
int32_t chorus_mfma_ceiling(int32_t normal_data, int32_t mix, int32_t launches, double* tflops, void* ws, size_t ws_bytes,
                            void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CHORUS_OPS_H */
