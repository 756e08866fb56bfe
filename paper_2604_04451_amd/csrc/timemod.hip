// Timestep injection (Sec. 2.1, Fig. 2): the projected timestep embedding of one denoising step.
//   f = [cos(t w_i), sin(t w_i)], w_i = 10000^(-i / half)          sinusoidal features, freq_dim = 2 half
//   e = W2 silu(W1 f + b1) + b2                                     [D]
//   t_mod  = reshape(Wp silu(e) + bp, [6, D])                       modulation rows of every block
//   t_head = [e, e]                                                 the head adds e to both rows of its table
// Three matrix-vector products with bf16 weights and fp32 activations: HBM-bound on the weights
// (2 (D F + D D + 6 D D) bytes), one wave per output row, 16-byte weight loads.
#include "chorus_ops.h"
#include "common.h"

namespace chorus {
namespace {

__global__ __launch_bounds__(256) void sinusoid_kernel(float t, int half, float* __restrict__ f) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= half) return;
  const float w = exp2f(-(float)i / (float)half * 13.287712379549449f);  // 10000^(-i/half)
  float sn, cs;
  sincosf(t * w, &sn, &cs);
  f[i] = cs;
  f[half + i] = sn;
}

// out[n] = sum_k W[n][k] act(x[k]) + b[n]; ACT: silu on the input vector. One wave per row n; K % 8 == 0.
// out2 (optional) receives the same values (the two head rows).
template <bool SILU_IN>
__global__ __launch_bounds__(256) void gemv_bf16w_kernel(const uint16_t* __restrict__ W, const float* __restrict__ x,
                                                         const float* __restrict__ b, float* __restrict__ out,
                                                         float* __restrict__ out2, int N, int K) {
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= N) return;
  const uint16_t* w = W + (long)n * K;
  float acc = 0.f;
  for (int k = lane * 8; k < K; k += 64 * 8) {
    const u32x4 u = *reinterpret_cast<const u32x4*>(w + k);
    const f32x4 x0 = *reinterpret_cast<const f32x4*>(x + k);
    const f32x4 x1 = *reinterpret_cast<const f32x4*>(x + k + 4);
    float xv[8] = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float v = xv[j];
      if (SILU_IN) v = v / (1.0f + __expf(-v));
      const float wv = __uint_as_float((j & 1) ? (u[j >> 1] & 0xffff0000u) : (u[j >> 1] << 16));
      acc = __builtin_fmaf(wv, v, acc);
    }
  }
  acc = wave_sum(acc);
  if (lane == 0) {
    const float r = acc + (b ? b[n] : 0.f);
    out[n] = r;
    if (out2) out2[n] = r;
  }
}

}  // namespace
}  // namespace chorus

using namespace chorus;

extern "C" {

size_t chorus_time_mod_workspace_bytes(int32_t D, int32_t freq_dim) {
  if (D <= 0 || freq_dim <= 0) return 0;
  return align_up((size_t)freq_dim * 4, 256) + align_up((size_t)D * 4, 256);
}

int32_t chorus_time_mod(float t, int32_t freq_dim, int32_t D, const chorus_time_weights* w, float* t_mod, float* t_head,
                        void* ws, size_t ws_bytes, void* stream) {
  if (!w || !t_mod || !t_head || D <= 0 || freq_dim <= 0) return CHORUS_E_ARG;
  if (!w->w_t1 || !w->w_t2 || !w->w_tp) return CHORUS_E_ARG;
  if ((freq_dim & 7) != 0 || (D & 7) != 0) return CHORUS_E_SHAPE;
  if (!aligned16(w->w_t1) || !aligned16(w->w_t2) || !aligned16(w->w_tp) || !aligned16(t_mod) || !aligned16(t_head))
    return CHORUS_E_ARG;
  if (!ws || !aligned16(ws) || ws_bytes < chorus_time_mod_workspace_bytes(D, freq_dim)) return CHORUS_E_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  float* f = (float*)ws;
  float* h = (float*)((uint8_t*)ws + align_up((size_t)freq_dim * 4, 256));
  const int half = freq_dim / 2;
  hipLaunchKernelGGL(sinusoid_kernel, dim3((unsigned)((half + 255) / 256)), dim3(256), 0, s, t, half, f);
  CHORUS_LAUNCH_CHECK();
  // h = W1 f + b1;  e = W2 silu(h) + b2 -> both head rows;  t_mod = Wp silu(e) + bp
  hipLaunchKernelGGL(gemv_bf16w_kernel<false>, dim3((unsigned)((D + 3) / 4)), dim3(256), 0, s, w->w_t1, f, w->b_t1, h,
                     (float*)nullptr, D, freq_dim);
  CHORUS_LAUNCH_CHECK();
  hipLaunchKernelGGL(gemv_bf16w_kernel<true>, dim3((unsigned)((D + 3) / 4)), dim3(256), 0, s, w->w_t2, h, w->b_t2, t_head,
                     t_head + D, D, D);
  CHORUS_LAUNCH_CHECK();
  hipLaunchKernelGGL(gemv_bf16w_kernel<true>, dim3((unsigned)((6 * D + 3) / 4)), dim3(256), 0, s, w->w_tp, t_head, w->b_tp,
                     t_mod, (float*)nullptr, 6 * D, D);
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

}  // extern "C"
