// chorus_dit_block_step: one DiT block forward as a fixed sequence of the
// library's own kernels on the caller's stream (no host synchronisation, no
// allocation). Also the optional per-kernel event timing used by benchmarks.
#include <vector>

#include "chorus_ops.h"
#include "common.h"

namespace chorus {
namespace {

// Benchmark profiler (the library's only process-wide state; off by default, not thread-safe). Events come from a
// pool that survives chorus_prof_reset, so a warm-up pass with the profiler on creates them and the timed passes
// only record.
struct ProfRec {
  int cls;
  int ev;  // index of the start event in the pool; the stop event follows it
};
unsigned g_prof_mask = 0;  // bit c set: kernel class c is timed
std::vector<ProfRec> g_prof;
std::vector<hipEvent_t> g_prof_pool;
size_t g_prof_pool_used = 0;

struct ProfScope {
  hipStream_t s;
  ProfRec rec;
  bool live;
  ProfScope(int cls, hipStream_t st) : s(st), live(false) {
    if (!(g_prof_mask & (1u << cls))) return;
    while (g_prof_pool.size() < g_prof_pool_used + 2) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) return;
      g_prof_pool.push_back(e);
    }
    rec.cls = cls;
    rec.ev = (int)g_prof_pool_used;
    g_prof_pool_used += 2;
    hipEventRecord(g_prof_pool[rec.ev], s);
    live = true;
  }
  ~ProfScope() {
    if (!live) return;
    hipEventRecord(g_prof_pool[rec.ev + 1], s);
    g_prof.push_back(rec);
  }
};

struct BlockWs {
  uint16_t* h;      // [Ls, D]
  uint16_t* ao;     // [Ls, D]   attention output
  uint16_t* qkv;    // [Ls, 3D]  (region A start; the FFN hidden [Ls, F] aliases region A)
  uint16_t* qh;     // [H, Lpad, dh]
  uint16_t* kh;     // [H, Lpad, dh]
  uint16_t* vt;     // [D, Lpad]
  uint16_t* ffn;    // [Ls, F]
  uint16_t* tkv;    // [Lt, 2D]
  uint16_t* kc;     // [H, LtPad, dh]
  uint16_t* vct;    // [D, LtPad]
  size_t bytes;
};

inline long pad_rows(long L) { return (long)align_up((size_t)L, 256); }
inline long pad_text(long Lt) { return (long)align_up((size_t)Lt, 64); }

BlockWs carve(const chorus_block_shape& sh, long Ls, void* base) {
  const size_t D = sh.D, F = sh.F, Lt = sh.Lt;
  const size_t Lpad = pad_rows(Ls), LtPad = pad_text(Lt);
  const BytePtr p(base);
  size_t off = 0;
  auto take = [&](size_t elems) {
    uint16_t* r = (uint16_t*)(p + off);
    off += align_up(elems * 2, 256);
    return r;
  };
  BlockWs w;
  w.h = take(Ls * D);
  w.ao = take(Ls * D);
  size_t a0 = off;
  w.qkv = take(Ls * 3 * D);
  w.qh = take(Lpad * D);
  w.kh = take(Lpad * D);
  w.vt = take(Lpad * D);
  size_t a_bytes = off - a0;
  w.ffn = w.qkv;
  size_t ffn_bytes = align_up(Ls * F * 2, 256);
  if (ffn_bytes > a_bytes) off = a0 + ffn_bytes;
  w.tkv = take(Lt * 2 * D);
  w.kc = take(LtPad * D);
  w.vct = take(LtPad * D);
  w.bytes = off;
  return w;
}

int32_t check_shape(const chorus_block_shape* sh) {
  if (!sh) return CHORUS_E_ARG;
  if (sh->D <= 0 || sh->H <= 0 || sh->F <= 0 || sh->Lt < 1) return CHORUS_E_SHAPE;
  if ((sh->dh != 64 && sh->dh != 128) || sh->H * sh->dh != sh->D) return CHORUS_E_SHAPE;
  if (sh->D % 64 || sh->F % 64) return CHORUS_E_SHAPE;
  if (sh->gT <= 0 || sh->gH <= 0 || sh->gW <= 0) return CHORUS_E_SHAPE;
  return CHORUS_OK;
}

// cached text K / V of one block: K head-major [H, LtPad, dh], then V^T [D, LtPad], each padded to 256 bytes
inline size_t text_kv_half_bytes(const chorus_block_shape& sh) { return align_up((size_t)pad_text(sh.Lt) * sh.D * 2, 256); }

#define CHK(call)                   \
  do {                              \
    int32_t st__ = (call);          \
    if (st__ != CHORUS_OK) return st__; \
  } while (0)

}  // namespace
}  // namespace chorus

using namespace chorus;

extern "C" {

int32_t chorus_prof_enable(int32_t class_mask) {
  g_prof_mask = (unsigned)class_mask & ((1u << CHORUS_PROF_CLASSES) - 1u);
  return CHORUS_OK;
}

int32_t chorus_prof_reset(void) {
  g_prof.clear();  // the events stay in the pool for the next pass
  g_prof_pool_used = 0;
  return CHORUS_OK;
}

int32_t chorus_prof_read(int32_t kernel_class, double* total_ms, int32_t* launches) {
  if (!total_ms || !launches) return CHORUS_E_ARG;
  double tot = 0.0;
  int n = 0;
  for (auto& r : g_prof) {
    if (r.cls != kernel_class) continue;
    CHORUS_HIP(hipEventSynchronize(g_prof_pool[r.ev + 1]));
    float ms = 0.f;
    CHORUS_HIP(hipEventElapsedTime(&ms, g_prof_pool[r.ev], g_prof_pool[r.ev + 1]));
    tot += ms;
    ++n;
  }
  *total_ms = tot;
  *launches = n;
  return CHORUS_OK;
}

size_t chorus_dit_block_workspace_bytes(const chorus_block_shape* shape, int64_t Ls) {
  if (check_shape(shape) != CHORUS_OK || Ls < 0) return 0;
  return carve(*shape, Ls > 0 ? Ls : 1, nullptr).bytes;
}

}  // extern "C"

namespace chorus {
namespace {

// text K (normalised, head-major) and V^T of one block from the projected prompt embedding (cross-attention keys and
// values depend only on the prompt, Sec. 2.1, so one projection serves every denoising step of a request)
int32_t project_text_kv(const chorus_block_shape& sh, const chorus_block_weights* w, const uint16_t* text_ctx, uint16_t* tkv,
                        uint16_t* kc, uint16_t* vct, void* stream) {
  const int D = sh.D, H = sh.H, dh = sh.dh, Lt = sh.Lt;
  const long LtPad = pad_text(Lt);
  hipStream_t s = (hipStream_t)stream;
  {
    ProfScope p(CHORUS_PROF_GEMM, s);
    CHK(chorus_gemm_bf16(text_ctx, w->w_ckv, Lt, 2 * D, D, CHORUS_EPI_BF16, tkv, w->b_ckv, nullptr, nullptr, 1.f, stream));
  }
  {
    ProfScope p(CHORUS_PROF_NORM, s);
    CHK(chorus_qk_norm_rope(tkv, 2L * D, w->g_ck, kc, Lt, LtPad, H, dh, nullptr, sh.gT, sh.gH, sh.gW, 0, 1.0f, stream));
    CHK(chorus_v_transpose(tkv + D, 2L * D, vct, Lt, LtPad, D, stream));
  }
  return CHORUS_OK;
}

// one block; exactly one of text_ctx (project K / V here) and text_kv (use the cached projection) is given
int32_t block_step_impl(const chorus_block_shape* shape, const chorus_block_weights* w, float* x, int64_t Ls,
                        const int32_t* token_idx, const uint16_t* text_ctx, const uint16_t* text_kv, const float* t_mod,
                        const float* tgaa_key_scale, float gamma_o, void* ws, size_t ws_bytes, void* stream) {
  CHK(check_shape(shape));
  if (Ls < 0) return CHORUS_E_ARG;
  if (Ls == 0) return CHORUS_OK;
  if (!w || !x || (!text_ctx && !text_kv) || !t_mod) return CHORUS_E_ARG;
  const chorus_block_shape& sh = *shape;
  if (Ls > (int64_t)sh.gT * sh.gH * sh.gW && token_idx == nullptr) return CHORUS_E_SHAPE;
  if (!ws) return CHORUS_E_WORKSPACE;
  if (!aligned16(ws) || !aligned16(x) || !aligned16(text_ctx) || !aligned16(text_kv) || !aligned16(t_mod) ||
      !aligned16(tgaa_key_scale))
    return CHORUS_E_ARG;
  BlockWs b = carve(sh, Ls, ws);
  if (ws_bytes < b.bytes) return CHORUS_E_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const int D = sh.D, F = sh.F, H = sh.H, dh = sh.dh, Lt = sh.Lt;
  const long Lpad = pad_rows(Ls), LtPad = pad_text(Lt);
  const float* tab = w->mod_table;
  auto row = [&](const float* base, int r) { return base + (size_t)r * D; };

  // 1. AdaLN modulation -> QKV projection
  {
    ProfScope p(CHORUS_PROF_NORM, s);
    CHK(chorus_ln_modulate(x, b.h, Ls, D, row(tab, 1), row(t_mod, 1), row(tab, 0), row(t_mod, 0), 1, stream));
  }
  {
    ProfScope p(CHORUS_PROF_GEMM, s);
    CHK(chorus_gemm_bf16(b.h, w->w_qkv, Ls, 3 * D, D, CHORUS_EPI_BF16, b.qkv, w->b_qkv, nullptr, nullptr, 1.f, stream));
  }
  // 2-3. q/k RMSNorm + RoPE into head-major layout; V into key-contiguous layout.
  // Attention over 512 keys or more without a column scale runs the kernel that takes its queries already multiplied by
  // log2(e) / sqrt(dh): the factor enters here, in fp32 ahead of the one rounding to bf16 (the same condition as
  // chorus_attention's default choice).
  const bool q_prescaled = CHORUS_ATTENTION_LONG_KEYS(Ls, Lpad);
  {
    ProfScope p(CHORUS_PROF_NORM, s);
    CHK(chorus_qk_norm_rope(b.qkv, 3L * D, w->g_q, b.qh, Ls, Lpad, H, dh, token_idx, sh.gT, sh.gH, sh.gW, 1,
                            q_prescaled ? CHORUS_ATTENTION_Q_PRESCALE(dh) : 1.0f, stream));
    CHK(chorus_qk_norm_rope(b.qkv + D, 3L * D, w->g_k, b.kh, Ls, Lpad, H, dh, token_idx, sh.gT, sh.gH, sh.gW, 1, 1.0f, stream));
    CHK(chorus_v_transpose(b.qkv + 2 * D, 3L * D, b.vt, Ls, Lpad, D, stream));
  }
  // 4. self-attention over exactly the Ls rows, output projection, gated residual
  {
    ProfScope p(CHORUS_PROF_SELF_ATTN, s);
    CHK(chorus_attention(b.qh, b.kh, b.vt, b.ao, nullptr, Ls, Ls, Lpad, Lpad, H, dh, q_prescaled ? 6 : 0, stream));
  }
  {
    ProfScope p(CHORUS_PROF_GEMM, s);
    CHK(chorus_gemm_bf16(b.ao, w->w_o, Ls, D, D, CHORUS_EPI_RESID, x, w->b_o, row(tab, 2), row(t_mod, 2), 1.f, stream));
  }
  // 5. cross-attention with TGAA
  {
    ProfScope p(CHORUS_PROF_NORM, s);
    CHK(chorus_ln_modulate(x, b.h, Ls, D, w->ln3_w, nullptr, w->ln3_b, nullptr, 0, stream));
  }
  {
    ProfScope p(CHORUS_PROF_GEMM, s);
    CHK(chorus_gemm_bf16(b.h, w->w_cq, Ls, D, D, CHORUS_EPI_BF16, b.qkv, w->b_cq, nullptr, nullptr, 1.f, stream));
  }
  const uint16_t* kc = b.kc;
  const uint16_t* vct = b.vct;
  if (text_kv) {
    kc = text_kv;
    vct = text_kv + text_kv_half_bytes(sh) / 2;
  } else {
    CHK(project_text_kv(sh, w, text_ctx, b.tkv, b.kc, b.vct, stream));
  }
  // cross-attention over 512 text tokens or more: pre-scaled queries as above, with or without a TGAA factor
  const bool cq_prescaled = CHORUS_ATTENTION_LONG_KEYS(Lt, LtPad);
  {
    ProfScope p(CHORUS_PROF_NORM, s);
    CHK(chorus_qk_norm_rope(b.qkv, D, w->g_cq, b.qh, Ls, Lpad, H, dh, nullptr, sh.gT, sh.gH, sh.gW, 0,
                            cq_prescaled ? CHORUS_ATTENTION_Q_PRESCALE(dh) : 1.0f, stream));
  }
  {
    ProfScope p(CHORUS_PROF_CROSS_ATTN, s);
    CHK(chorus_attention(b.qh, kc, vct, b.ao, tgaa_key_scale, Ls, Lt, Lpad, LtPad, H, dh, cq_prescaled ? 6 : 0, stream));
  }
  {
    ProfScope p(CHORUS_PROF_GEMM, s);
    CHK(chorus_gemm_bf16(b.ao, w->w_co, Ls, D, D, CHORUS_EPI_RESID, x, w->b_co, nullptr, nullptr, gamma_o, stream));
  }
  // 6. FFN
  {
    ProfScope p(CHORUS_PROF_NORM, s);
    CHK(chorus_ln_modulate(x, b.h, Ls, D, row(tab, 4), row(t_mod, 4), row(tab, 3), row(t_mod, 3), 1, stream));
  }
  {
    ProfScope p(CHORUS_PROF_GEMM, s);
    CHK(chorus_gemm_bf16(b.h, w->w_1, Ls, F, D, CHORUS_EPI_GELU_BF16, b.ffn, w->b_1, nullptr, nullptr, 1.f, stream));
    CHK(chorus_gemm_bf16(b.ffn, w->w_2, Ls, D, F, CHORUS_EPI_RESID, x, w->b_2, row(tab, 5), row(t_mod, 5), 1.f, stream));
  }
  return CHORUS_OK;
}

}  // namespace
}  // namespace chorus

extern "C" {

int32_t chorus_dit_block_step(const chorus_block_shape* shape, const chorus_block_weights* w, float* x, int64_t Ls,
                              const int32_t* token_idx, const uint16_t* text_ctx, const float* t_mod,
                              const float* tgaa_key_scale, float gamma_o, void* ws, size_t ws_bytes, void* stream) {
  if (Ls > 0 && !text_ctx) return CHORUS_E_ARG;
  return block_step_impl(shape, w, x, Ls, token_idx, text_ctx, nullptr, t_mod, tgaa_key_scale, gamma_o, ws, ws_bytes, stream);
}

int32_t chorus_dit_block_step_kv(const chorus_block_shape* shape, const chorus_block_weights* w, float* x, int64_t Ls,
                                 const int32_t* token_idx, const uint16_t* text_kv, const float* t_mod,
                                 const float* tgaa_key_scale, float gamma_o, void* ws, size_t ws_bytes, void* stream) {
  if (Ls > 0 && !text_kv) return CHORUS_E_ARG;
  return block_step_impl(shape, w, x, Ls, token_idx, nullptr, text_kv, t_mod, tgaa_key_scale, gamma_o, ws, ws_bytes, stream);
}

size_t chorus_text_kv_bytes(const chorus_block_shape* shape) {
  if (check_shape(shape) != CHORUS_OK) return 0;
  return 2 * text_kv_half_bytes(*shape);
}

size_t chorus_text_kv_workspace_bytes(const chorus_block_shape* shape) {
  if (check_shape(shape) != CHORUS_OK) return 0;
  return align_up((size_t)shape->Lt * 2 * shape->D * 2, 256);
}

int32_t chorus_text_kv_project(const chorus_block_shape* shape, const chorus_block_weights* w, const uint16_t* text_ctx,
                               uint16_t* text_kv, void* ws, size_t ws_bytes, void* stream) {
  CHK(check_shape(shape));
  if (!w || !text_ctx || !text_kv) return CHORUS_E_ARG;
  if (!aligned16(text_ctx) || !aligned16(text_kv) || !aligned16(ws)) return CHORUS_E_ARG;
  if (!ws || ws_bytes < chorus_text_kv_workspace_bytes(shape)) return CHORUS_E_WORKSPACE;
  return project_text_kv(*shape, w, text_ctx, (uint16_t*)ws, text_kv, text_kv + text_kv_half_bytes(*shape) / 2, stream);
}

}  // extern "C"
