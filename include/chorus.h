/*
 * chorus.h -- C ABI of the Chorus hot path for AMD MI355X (gfx950).
 *
 * Chorus (three-stage inter-request caching for video DiT serving) splits an
 * N-step denoise into full reuse of a cached request's latent (stage 1),
 * selective region denoising (stage 2) and full computation (stage 3). This
 * library holds the data-parallel part: the cache lookup, the stage schedule,
 * the DiT block forward with Token-Guided Attention Amplification (TGAA), the
 * token compaction that makes skipped regions free, and the latent fusion.
 *
 * Conventions
 *  - Every function returns an int32 status: CHORUS_OK or a negative error.
 *    No function throws, aborts or allocates device memory.
 *  - "dev" pointers are device pointers owned by the caller; "host" pointers
 *    are ordinary host memory. All tensors are row-major and 16-byte aligned.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Device work is enqueued on it and the call returns without waiting.
 *  - bf16 tensors are passed as uint16_t bit patterns.
 *  - Workspaces are caller-provided device buffers; the *_workspace_bytes
 *    functions give the size. A workspace holds no state between calls.
 *  - Weight matrices are [out_features, in_features] (y = x W^T + b).
 */
#ifndef CHORUS_H
#define CHORUS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CHORUS_OK            0
#define CHORUS_E_ARG        (-1) /* null or misaligned pointer, negative size */
#define CHORUS_E_SHAPE      (-2) /* dimensions the kernels do not support */
#define CHORUS_E_WORKSPACE  (-3) /* workspace missing or too small */
#define CHORUS_E_HIP        (-4) /* a HIP call failed; see chorus_last_hip_error */

/* Library version (major*10000 + minor*100 + patch). Host only. */
int32_t chorus_version(void);
/* hipError_t of the last failed HIP call made by this library on the calling thread (0 if none). */
int32_t chorus_last_hip_error(void);

/* ------------------------------------------------------------------------
 * Stage-1 retrieval (Sec. 3.1 "Full Reuse"; appendix "cache backend"):
 * top-1 cosine similarity of the target prompt embedding against the cached
 * prompt embeddings; the request is a hit when the score m reaches tau
 * (the fallback rule of Sec. 3.1 is m < tau).
 *   cache_emb  dev  [N, d] fp32 (rows need not be unit norm)
 *   query      dev  [d]    fp32
 *   out        dev  one chorus_lookup_result
 *   ws         dev  chorus_cache_lookup_workspace_bytes(N) bytes
 * Scores are computed in fp32 with one fixed summation order per row, so equal
 * rows get equal scores; the lowest index wins ties. A zero-norm row or query
 * scores -inf. N == 0 gives index -1, score -inf, hit 0. d must be a multiple of 4;
 * N at most 2^31 - 2 (the index is an int32), CHORUS_E_SHAPE beyond.
 * Two launches: the scan leaves one (best value, index) pair per workgroup in ws, a single
 * workgroup picks among them.
 * ------------------------------------------------------------------------ */
typedef struct {
  int32_t index;
  float score;
  int32_t hit;
} chorus_lookup_result;

size_t chorus_cache_lookup_workspace_bytes(int64_t N);
int32_t chorus_cache_lookup(const float* cache_emb, int64_t N, int32_t d, const float* query, float tau,
                            chorus_lookup_result* out, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * chorus_cache_lookup for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * allocation. Same arguments (minus the workspace), same kernels, bit-identical result. The
 * scan's per-workgroup partial results live in a 33 KB array in the library's own device
 * image (one copy per GPU, held until the process ends) instead of a caller buffer. The call
 * makes no hipMalloc / hipFree and no allocating library call; the first call on a device
 * resolves the array's address there (make that call outside graph capture).
 * All calls on one GPU share that array: calls that overlap in time on one GPU (two streams,
 * two threads) race and may return each other's result; calls on one stream, or otherwise
 * ordered, are safe, and nothing a call leaves in the array is read by the next.
 * Limits: N at most 2^31 - 2 as for chorus_cache_lookup (the array serves every such N, the
 * scan never uses more than 4096 workgroups); device ordinals 0..63. CHORUS_E_SHAPE beyond.
 * ------------------------------------------------------------------------ */
int32_t chorus_cache_lookup_static(const float* cache_emb, int64_t N, int32_t d, const float* query, float tau,
                                   chorus_lookup_result* out, void* stream);

/* ------------------------------------------------------------------------
 * The same retrieval over a low-precision copy of the cached embeddings (cache maintenance
 * around Sec. 3.1 "Full Reuse"; the appendix's cache backend): the scan reads bf16 rows (half
 * the bytes of the fp32 scan) or FP8 E4M3 rows (a quarter); every row whose approximate score
 * lies within a margin of the best approximate score is then re-scored from its fp32 row, and
 * the best of those is returned. The margin is twice the most a cosine can move when a row is
 * replaced by its low-precision copy (bf16: every element within 2^-8 of itself; FP8: 2^-4,
 * and 2^-10 of the scaled row's largest magnitude / 448 below 2^-6), so the true best row is
 * always re-scored: index, score and hit are chorus_cache_lookup's, bit for bit.
 *   chorus_cache_lowprec_bytes   device bytes of the copy of N rows (N d elements of 2 or 1 bytes)
 *   chorus_cache_lowprec_store   encodes n_rows fp32 rows (emb dev [n_rows, d]) into out dev
 *                                [n_rows, d]; call it on the whole cache once and on an entry's
 *                                row after chorus_cache_insert. bf16: round to nearest even.
 *                                FP8: the row times 448 / max|row| (two fp32 operations), rounded
 *                                to nearest even; the scale is not kept (a cosine does not
 *                                depend on it); an all-zero row encodes as zeros.
 *   chorus_cache_lookup_lowprec  cache_emb dev [N, d] fp32 (read only for the re-scored rows),
 *                                cache_lp dev [N, d] codes, n_rescored dev int32 or NULL (the
 *                                number of rows re-scored), ws dev of
 *                                chorus_cache_lookup_lowprec_workspace_bytes(N) bytes.
 * d a multiple of 16; N at most 2^31 - 2. Three launches: the low-precision scan, the re-rank
 * (in the scan's launch shape: when every row is a candidate, as with FP8 on a query far from
 * every entry, it costs one fp32 scan; usually one wave has work) and a single-workgroup pick.
 * Errors: CHORUS_E_ARG (null / misaligned pointer, unknown format), CHORUS_E_SHAPE,
 * CHORUS_E_WORKSPACE, CHORUS_E_HIP.
 * ------------------------------------------------------------------------ */
#define CHORUS_LP_BF16 0
#define CHORUS_LP_FP8 1
size_t chorus_cache_lowprec_bytes(int64_t N, int32_t d, int32_t format);
int32_t chorus_cache_lowprec_store(const float* emb, int64_t n_rows, int32_t d, int32_t format, void* out, void* stream);
size_t chorus_cache_lookup_lowprec_workspace_bytes(int64_t N);
int32_t chorus_cache_lookup_lowprec(const float* cache_emb, const void* cache_lp, int32_t format, int64_t N, int32_t d,
                                    const float* query, float tau, chorus_lookup_result* out, int32_t* n_rescored, void* ws,
                                    size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * The same retrieval for a batch of queued requests, with candidates: the k best entries
 * by cosine similarity for each of Q prompt embeddings. The cache is streamed once per 32
 * queries (a [N, d] x [d, Q] fp32 contraction on the matrix pipe), not once per query.
 *   queries    dev [Q, d] fp32
 *   out_index  dev [Q, k] int32, out_score dev [Q, k] fp32: descending score, equal scores
 *              by ascending index; positions beyond N hold index -1 and score -inf
 *   out_hit    dev [Q] int32: out_score[q, 0] >= tau
 *   ws         dev, chorus_cache_lookup_batch_workspace_bytes(N, d, Q) bytes
 * Scores are fp32 with a summation order that depends only on (N, d), not on the row, so
 * equal rows get equal scores; zero-norm rows or queries score -inf. Column 0 agrees with
 * chorus_cache_lookup up to the fp32 rounding of a different summation order.
 * 1 <= k <= 1024; d a multiple of 4; N < 2^31 - 256; Q == 0 is a no-op.
 * Errors: CHORUS_E_ARG, CHORUS_E_SHAPE, CHORUS_E_WORKSPACE, CHORUS_E_HIP.
 * ------------------------------------------------------------------------ */
size_t chorus_cache_lookup_batch_workspace_bytes(int64_t N, int32_t d, int32_t Q);
int32_t chorus_cache_lookup_batch(const float* cache_emb, int64_t N, int32_t d, const float* queries, int32_t Q, float tau,
                                  int32_t k, int32_t* out_index, float* out_score, int32_t* out_hit, void* ws,
                                  size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Cache update (Sec. 3.1 "Cache Update"): after a miss the request's prompt embedding and
 * an intermediate latent are stored for later requests. Two device copies, bit for bit.
 *   cache_emb      dev [capacity, d] fp32, row `slot` is overwritten with emb [d]
 *   cache_latents  dev [capacity, latent_elems] fp32, row `slot` is overwritten with latent
 * Which entry to replace is the caller's policy. A never-written (all-zero) row scores
 * -inf in chorus_cache_lookup, so a zero-filled cache is an empty one.
 * Errors: CHORUS_E_ARG (null pointer, slot outside [0, capacity), d or latent_elems <= 0).
 * ------------------------------------------------------------------------ */
int32_t chorus_cache_insert(float* cache_emb, float* cache_latents, int64_t capacity, int64_t slot, int32_t d,
                            int64_t latent_elems, const float* emb, const float* latent, void* stream);

/* ------------------------------------------------------------------------
 * Stage boundaries (Eq. 1) and TGAA decay (Eq. 4). Host only.
 * The paper fixes properties, not formulas: 0 <= K1 <= K2 <= N, both monotone in
 * the matching score m, K1 = K2 = 0 when m < tau, amplification factors >= 1 that
 * fall with the step and with m. This map has them:
 *   s  = clip((m - tau)/(1 - tau), 0, 1)
 *   K1 = clip(floor(N (a1 + b1 s) + 1e-9), 0, N - r3)
 *   K2 = clip(K1 + floor(N (a2 + b2 s) + 1e-9), K1, N - r3)
 *   step i >= K1:  w = max(0, 1 - (i - K1)/max(1, K2 - K1)),
 *                  gamma_x = max(1, 1 + (Gamma_x - 1)(1 - lam s) w)
 * Steps below K1 are stage 1 (gamma reported as 1), below K2 stage 2, else stage 3.
 * gamma_override > 0 replaces both factors of the stage-2 steps.
 * params == NULL selects a1=b1=a2=b2=0.25, r3=1, Gamma_k=Gamma_o=1.5, lam=0.5.
 *   plan  host [N]; K1, K2 host (may be NULL)
 * ------------------------------------------------------------------------ */
typedef struct {
  double a1, b1, a2, b2;
  int32_t r3;
  double Gamma_k, Gamma_o, lam;
  double gamma_override;
} chorus_sched_params;

typedef struct {
  int32_t stage; /* 1, 2 or 3 */
  float gamma_k;
  float gamma_o;
} chorus_step_plan;

int32_t chorus_denoise_schedule(float m, float tau, int32_t N, const chorus_sched_params* params, int32_t* K1,
                                int32_t* K2, chorus_step_plan* plan);
/* The same schedule when the matched entry holds intermediate latents only at some depths
 * (Sec. 3.1 "Cache Update": the states after stored_steps[j] steps). Full reuse can only
 * resume from a stored state: K1 becomes the largest stored depth in [1, K1 of Eq. 1], K2 is
 * K1 plus the same region-stage length (clipped to N - r3), and *slot is that depth's
 * position in stored_steps. With no such depth (or on a miss) the plan is N plain steps,
 * K1 = K2 = 0 and *slot = -1.
 *   stored_steps host [n_stored] (any order; n_stored may be 0); slot host (may be NULL) */
int32_t chorus_denoise_schedule_stored(float m, float tau, int32_t N, const chorus_sched_params* params,
                                       const int32_t* stored_steps, int32_t n_stored, int32_t* K1, int32_t* K2,
                                       int32_t* slot, chorus_step_plan* plan);

/* ------------------------------------------------------------------------
 * One DiT block forward on Ls token rows, in place on the fp32 residual stream
 * (Sec. 2.1 and Fig. 2: self-attention, cross-attention on the prompt, timestep
 * injection, FFN; TGAA per Eq. 2 and Eq. 3). In stage 2 the caller passes only
 * the tokens selected by the visible mask (Sec. 3.3.3): self-attention runs over
 * exactly those Ls rows, so skipped regions cost nothing.
 *
 *   e = mod_table + t_mod -> (shift, scale, gate) for self-attention and FFN
 *   1. h = LN(x)(1 + scale_sa) + shift_sa; q,k,v = h Wqkv^T + b
 *   2. q, k RMS-normalised over all D (gains g_q, g_k); 3. 3-D RoPE on q, k at the
 *      token's original (t,h,w) (head dims split dh-4*(dh/6) | 2*(dh/6) | 2*(dh/6),
 *      pair (2p,2p+1) of a group of size g turns by pos * 10000^(-2p/g))
 *   4. x += gate_sa * (softmax(q k^T / sqrt(dh)) v Wo^T + bo)
 *   5. hc = LN(x) ln3_w + ln3_b; qc = RMS(hc Wcq^T + b); kc = RMS(ctx Wck^T + b);
 *      vc = ctx Wcv^T + b; logits_ij = tgaa_key_scale[j] (qc_i . kc_j)/sqrt(dh)
 *      (Eq. 2: keys of the differential tokens scaled by gamma_k, after the norm);
 *      x += gamma_o * (softmax(logits) vc Wco^T + bco)            (Eq. 3)
 *   6. x += gate_ffn * (gelu_tanh(LN(x)(1+scale_ffn)+shift_ffn) W1^T + b1) W2^T + b2)
 * LayerNorm/RMSNorm eps 1e-6. GEMM and attention operands are rounded to bf16,
 * accumulation and all normalisation / softmax / residual arithmetic is fp32.
 *
 *   x          dev [Ls, D] fp32, in/out
 *   token_idx  dev [Ls] int32 original token ids on the (gT,gH,gW) grid, ascending;
 *              NULL = identity
 *   text_ctx   dev [Lt, D] bf16, already projected to D
 *   t_mod      dev [6, D] fp32 projected timestep embedding
 *   tgaa_key_scale dev [Lt] fp32, 16-byte aligned (gamma_k on the differential tokens,
 *              1 elsewhere); NULL = all 1
 *   gamma_o    output amplification; 1 = neutral
 * Supported: dh in {64, 128}, H*dh == D, D % 64 == 0, F % 64 == 0, Lt >= 1.
 * Ls == 0 is a no-op.
 * ------------------------------------------------------------------------ */
typedef struct {
  int32_t D, H, dh, F, Lt;
  int32_t gT, gH, gW; /* token grid */
} chorus_block_shape;

typedef struct {
  const float* mod_table;  /* [6, D]: shift_sa, scale_sa, gate_sa, shift_ffn, scale_ffn, gate_ffn */
  const uint16_t* w_qkv;   /* [3D, D] bf16 */
  const float* b_qkv;      /* [3D] */
  const float* g_q;        /* [D] */
  const float* g_k;        /* [D] */
  const uint16_t* w_o;     /* [D, D] */
  const float* b_o;        /* [D] */
  const float* ln3_w;      /* [D] */
  const float* ln3_b;      /* [D] */
  const uint16_t* w_cq;    /* [D, D] */
  const float* b_cq;       /* [D] */
  const uint16_t* w_ckv;   /* [2D, D]: key rows then value rows */
  const float* b_ckv;      /* [2D] */
  const float* g_cq;       /* [D] */
  const float* g_ck;       /* [D] */
  const uint16_t* w_co;    /* [D, D] */
  const float* b_co;       /* [D] */
  const uint16_t* w_1;     /* [F, D] */
  const float* b_1;        /* [F] */
  const uint16_t* w_2;     /* [D, F] */
  const float* b_2;        /* [D] */
} chorus_block_weights;

size_t chorus_dit_block_workspace_bytes(const chorus_block_shape* shape, int64_t Ls);
int32_t chorus_dit_block_step(const chorus_block_shape* shape, const chorus_block_weights* w, float* x, int64_t Ls,
                              const int32_t* token_idx, const uint16_t* text_ctx, const float* t_mod,
                              const float* tgaa_key_scale, float gamma_o, void* ws, size_t ws_bytes, void* stream);

/* -----------------------------------------------------------------------------
 * Text keys / values of one block, projected once per request (Sec. 2.1: cross-attention
 * conditions on the prompt only, so its keys and values are the same at every denoising
 * step; Eq. 2 scales logits, not the stored keys, so TGAA leaves them valid).
 *   chorus_text_kv_bytes            device bytes of one block's entry: the normalised keys
 *                                   head-major [H, LtPad, dh] bf16, then the values
 *                                   key-contiguous [D, LtPad] bf16 (LtPad = Lt rounded up to 64)
 *   chorus_text_kv_workspace_bytes  scratch of chorus_text_kv_project ([Lt, 2D] bf16)
 *   chorus_text_kv_project          text_ctx dev [Lt, D] bf16 -> text_kv dev (caller-owned)
 *   chorus_dit_block_step_kv        chorus_dit_block_step with text_kv in place of text_ctx:
 *                                   the same kernels on the same values, so the result is
 *                                   bit-identical to the call that projects inside the block
 * Errors as chorus_dit_block_step. Asynchronous on `stream`, no allocation.
 * --------------------------------------------------------------------------- */
size_t chorus_text_kv_bytes(const chorus_block_shape* shape);
size_t chorus_text_kv_workspace_bytes(const chorus_block_shape* shape);
int32_t chorus_text_kv_project(const chorus_block_shape* shape, const chorus_block_weights* w, const uint16_t* text_ctx,
                               uint16_t* text_kv, void* ws, size_t ws_bytes, void* stream);
int32_t chorus_dit_block_step_kv(const chorus_block_shape* shape, const chorus_block_weights* w, float* x, int64_t Ls,
                                 const int32_t* token_idx, const uint16_t* text_kv, const float* t_mod,
                                 const float* tgaa_key_scale, float gamma_o, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Latent fusion (Eq. 6): out = M_edit * L + (1 - M_edit) * SL with a binary mask
 * given per token and expanded over channels and the ph x pw patch. Done as a
 * select, so it is exact and an all-zero mask returns SL bit for bit (stage-1
 * full reuse), an all-one mask returns L.
 *   out, L, SL  dev [C, T, H, W] fp32; out may alias L or SL
 *   mask_edit   dev [T, H/ph, W/pw] uint8, non-zero = keep the computed L
 * H % ph == 0, W % pw == 0.
 * ------------------------------------------------------------------------ */
int32_t chorus_region_blend(float* out, const float* L, const float* SL, const uint8_t* mask_edit, int32_t C,
                            int32_t T, int32_t H, int32_t W, int32_t ph, int32_t pw, void* stream);

/* ------------------------------------------------------------------------
 * Region selection helpers (Sec. 3.3.3: the masked tokens are selected before the
 * blocks run instead of being zeroed inside them).
 * compact: idx_out[0..count) = ascending positions n with mask[n] != 0.
 *   mask dev [L] uint8; idx_out dev [L] int32 (entries past count untouched);
 *   count_out dev int32. L <= 2^31-1. ws: chorus_region_compact_workspace_bytes(L).
 * gather:  dst[i, :] = src[idx[i], :]    scatter: dst[idx[i], :] = src[i, :]
 *   rows of row_bytes bytes (multiple of 4); idx dev [Ls] int32, distinct for scatter.
 * ------------------------------------------------------------------------ */
size_t chorus_region_compact_workspace_bytes(int64_t L);
int32_t chorus_region_compact(const uint8_t* mask, int64_t L, int32_t* idx_out, int32_t* count_out, void* ws,
                              size_t ws_bytes, void* stream);
int32_t chorus_region_gather_rows(void* dst, const void* src, const int32_t* idx, int64_t Ls, int64_t row_bytes,
                                  void* stream);
int32_t chorus_region_scatter_rows(void* dst, const void* src, const int32_t* idx, int64_t Ls, int64_t row_bytes,
                                   void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CHORUS_H */
