// Row-wise normalisation kernels of the DiT block (HBM-bound, fp32 arithmetic):
//  - LayerNorm + AdaLN modulation / affine, fp32 residual stream -> bf16 GEMM operand
//  - RMSNorm over the full width + 3-D RoPE, token-major bf16 -> head-major bf16
//  - V transpose into the key-contiguous layout the attention kernel reads
#include "chorus_ops.h"
#include "common.h"

namespace chorus {
namespace {

constexpr float kEps = 1e-6f;

// One wave per row. NV > 0: D == NV*256 and the row lives in registers (one HBM
// read). NV == 0: any D % 4 == 0, the row is re-read from cache for each pass.
template <int NV>
__global__ __launch_bounds__(256) void ln_modulate_kernel(const float* __restrict__ x, uint16_t* __restrict__ out,
                                                          long L, int D, const float* __restrict__ mul0,
                                                          const float* __restrict__ mul1,
                                                          const float* __restrict__ add0,
                                                          const float* __restrict__ add1, float mul_base) {
  // the two modulation vectors are the same for every row: the workgroup combines them once into LDS
  // ((base + mul0 + mul1) and (add0 + add1)) while the rows' loads are in flight
  extern __shared__ __attribute__((aligned(16))) float s_tab[];  // [2][D]
  const int lane = threadIdx.x & 63;
  const long row_raw = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const bool live = row_raw < L;
  const long row = live ? row_raw : L - 1;  // a wave past the end keeps the barrier company and stores nothing
  const float4* xr = reinterpret_cast<const float4*>(x + row * (long)D);
  const int n4 = D >> 2;
  const float invD = 1.0f / (float)D;
  float mean, rstd;
  float4 v[NV > 0 ? NV : 1];
  if (NV > 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] = xr[lane + 64 * i];
  }
  {
    const float4* m0 = reinterpret_cast<const float4*>(mul0);
    const float4* m1 = reinterpret_cast<const float4*>(mul1);
    const float4* a0 = reinterpret_cast<const float4*>(add0);
    const float4* a1 = reinterpret_cast<const float4*>(add1);
    for (int i = threadIdx.x; i < n4; i += 256) {
      float4 mu = m0[i];
      mu.x += mul_base; mu.y += mul_base; mu.z += mul_base; mu.w += mul_base;
      if (mul1) {
        const float4 e = m1[i];
        mu.x += e.x; mu.y += e.y; mu.z += e.z; mu.w += e.w;
      }
      float4 ad = a0[i];
      if (add1) {
        const float4 e = a1[i];
        ad.x += e.x; ad.y += e.y; ad.z += e.z; ad.w += e.w;
      }
      reinterpret_cast<float4*>(s_tab)[i] = mu;
      reinterpret_cast<float4*>(s_tab + D)[i] = ad;
    }
  }
  if (NV > 0) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    mean = wave_sum(s) * invD;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      float a = v[i].x - mean, b = v[i].y - mean, c = v[i].z - mean, d = v[i].w - mean;
      q += (a * a + b * b) + (c * c + d * d);
    }
    rstd = rsqrtf(wave_sum(q) * invD + kEps);
  } else {
    float s = 0.f;
    for (int i = lane; i < n4; i += 64) {
      float4 t = xr[i];
      s += (t.x + t.y) + (t.z + t.w);
    }
    mean = wave_sum(s) * invD;
    float q = 0.f;
    for (int i = lane; i < n4; i += 64) {
      float4 t = xr[i];
      float a = t.x - mean, b = t.y - mean, c = t.z - mean, d = t.w - mean;
      q += (a * a + b * b) + (c * c + d * d);
    }
    rstd = rsqrtf(wave_sum(q) * invD + kEps);
  }
  __syncthreads();  // the combined vectors are in LDS
  if (!live) return;
  uint2* orow = reinterpret_cast<uint2*>(out + row * (long)D);
  const int iters = NV > 0 ? NV : (n4 + 63) / 64;
#pragma unroll
  for (int it = 0; it < iters; ++it) {
    int i = lane + 64 * it;
    if (NV == 0 && i >= n4) break;
    float4 t = NV > 0 ? v[NV > 0 ? it : 0] : xr[i];
    const float4 mu = reinterpret_cast<const float4*>(s_tab)[i];
    const float4 ad = reinterpret_cast<const float4*>(s_tab + D)[i];
    float r0 = (t.x - mean) * rstd * mu.x + ad.x;
    float r1 = (t.y - mean) * rstd * mu.y + ad.y;
    float r2 = (t.z - mean) * rstd * mu.z + ad.z;
    float r3 = (t.w - mean) * rstd * mu.w + ad.w;
    orow[i] = make_uint2(pack_bf16x2(r0, r1), pack_bf16x2(r2, r3));
  }
}

// One wave per token row (rows >= L up to Lpad are written as zeros). Lanes own
// 8-element chunks; chunk c covers dims [8c, 8c+8) of the D-wide row, inside one head.
// NCH > 0: D == 512 * NCH and the row lives in registers: its loads are issued first, the rotation
// angles are computed while they are in flight, and the row is read from HBM once. NCH == 0: any D % 8 == 0,
// the row is read again (from cache) for the second pass.
template <int NCH>
__global__ __launch_bounds__(256) void qk_norm_rope_kernel(const uint16_t* __restrict__ in, long ld,
                                                           const float* __restrict__ gain, uint16_t* __restrict__ out,
                                                           long L, long Lpad, int H, int dh,
                                                           const int* __restrict__ token_idx, int gH, int gW,
                                                           int rope, float out_scale) {
  __shared__ float s_cos[4][64];
  __shared__ float s_sin[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const long row = (long)blockIdx.x * 4 + wave;
  if (row >= Lpad) return;
  const int D = H * dh;
  const int nchunk = D >> 3;
  if (row >= L) {
    for (int c = lane; c < nchunk; c += 64) {
      int head = (c * 8) / dh, d0 = (c * 8) % dh;
      *reinterpret_cast<uint4*>(out + ((long)head * Lpad + row) * dh + d0) = make_uint4(0, 0, 0, 0);
    }
    return;
  }
  const uint16_t* r = in + row * ld;
  u32x4 rv[NCH > 0 ? NCH : 1];
  if (NCH > 0) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) rv[i] = *reinterpret_cast<const u32x4*>(r + (lane + 64 * i) * 8);
  }
  if (rope) {
    // rotation angles depend on the pair index inside a head only: dh/2 <= 64 of them
    long n = token_idx ? (long)token_idx[row] : row;
    int pw = (int)(n % gW), phh = (int)((n / gW) % gH), pt = (int)(n / ((long)gW * gH));
    const int s6 = dh / 6;
    const int g0 = dh - 4 * s6, g1 = 2 * s6;
    if (lane < dh / 2) {
      int d = 2 * lane;
      int off, g, pos;
      if (d < g0) { off = 0; g = g0; pos = pt; }
      else if (d < g0 + g1) { off = g0; g = g1; pos = phh; }
      else { off = g0 + g1; g = g1; pos = pw; }
      float expo = -(float)(d - off) / (float)g;           // -2p/g
      float freq = exp2f(expo * 13.287712379549449f);       // 10000^expo
      float sn, cs;
      sincosf((float)pos * freq, &sn, &cs);
      s_cos[wave][lane] = cs;
      s_sin[wave][lane] = sn;
    }
    __builtin_amdgcn_wave_barrier();
  }
  // pass 1: mean of squares
  float ss = 0.f;
  if (NCH > 0) {
#pragma unroll
    for (int i = 0; i < NCH; ++i)
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        float a = __uint_as_float(rv[i][k] << 16), b = __uint_as_float(rv[i][k] & 0xffff0000u);
        ss += a * a + b * b;
      }
  } else {
    for (int c = lane; c < nchunk; c += 64) {
      uint4 u = *reinterpret_cast<const uint4*>(r + c * 8);
      uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        float a = __uint_as_float(w[k] << 16), b = __uint_as_float(w[k] & 0xffff0000u);
        ss += a * a + b * b;
      }
    }
  }
  const float rstd = rsqrtf(wave_sum(ss) / (float)D + kEps) * out_scale;
  const int iters = NCH > 0 ? NCH : (nchunk + 63) / 64;
#pragma unroll
  for (int it = 0; it < iters; ++it) {
    const int c = lane + 64 * it;
    if (NCH == 0 && c >= nchunk) break;
    u32x4 u;
    if (NCH > 0) u = rv[NCH > 0 ? it : 0];
    else u = *reinterpret_cast<const u32x4*>(r + c * 8);
    const uint32_t w[4] = {u[0], u[1], u[2], u[3]};
    const float4 ga = *reinterpret_cast<const float4*>(gain + c * 8);
    const float4 gb = *reinterpret_cast<const float4*>(gain + c * 8 + 4);
    const float gv[8] = {ga.x, ga.y, ga.z, ga.w, gb.x, gb.y, gb.z, gb.w};
    const int head = (c * 8) / dh, d0 = (c * 8) % dh;
    uint32_t o[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      float a = __uint_as_float(w[k] << 16) * rstd * gv[2 * k];
      float b = __uint_as_float(w[k] & 0xffff0000u) * rstd * gv[2 * k + 1];
      if (rope) {
        float cs = s_cos[wave][(d0 >> 1) + k], sn = s_sin[wave][(d0 >> 1) + k];
        float ra = a * cs - b * sn, rb = a * sn + b * cs;
        a = ra;
        b = rb;
      }
      o[k] = pack_bf16x2(a, b);
    }
    *reinterpret_cast<uint4*>(out + ((long)head * Lpad + row) * dh + d0) = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

// Tile transpose: in[token][dim] -> out[dim][pos], 64 tokens x 64 dims per workgroup.
// Inside every group of 16 tokens the output position p = 8c + 4u + i holds token
// 8u + 4c + i: that is the order in which a lane of the attention kernel holds its
// probabilities after the QK^T MFMA, so its V operand is one 16-byte read.
__global__ __launch_bounds__(256) void v_transpose_kernel(const uint16_t* __restrict__ in, long ld,
                                                          uint16_t* __restrict__ out, long L, long Lpad) {
  __shared__ uint16_t tile[64][64 + 2];
  const long t0 = (long)blockIdx.x * 64;
  const int d0 = blockIdx.y * 64;
  for (int q = threadIdx.x; q < 512; q += 256) {
    int tok = q >> 3, ch = q & 7;
    uint4 u = make_uint4(0, 0, 0, 0);
    if (t0 + tok < L) u = *reinterpret_cast<const uint4*>(in + (t0 + tok) * ld + d0 + ch * 8);
    uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      tile[tok][ch * 8 + 2 * k] = (uint16_t)(w[k] & 0xffffu);
      tile[tok][ch * 8 + 2 * k + 1] = (uint16_t)(w[k] >> 16);
    }
  }
  __syncthreads();
  for (int q = threadIdx.x; q < 512; q += 256) {
    int dim = q >> 3, pc = q & 7;  // 8 output positions [8pc, 8pc+8)
    uint16_t v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      int p = pc * 8 + e;
      int G = p >> 4, rr = p & 15;
      int c = rr >> 3, u = (rr >> 2) & 1, i = rr & 3;
      v[e] = tile[16 * G + 8 * u + 4 * c + i][dim];
    }
    uint4 o = make_uint4(v[0] | ((uint32_t)v[1] << 16), v[2] | ((uint32_t)v[3] << 16), v[4] | ((uint32_t)v[5] << 16),
                         v[6] | ((uint32_t)v[7] << 16));
    *reinterpret_cast<uint4*>(out + (long)(d0 + dim) * Lpad + t0 + pc * 8) = o;
  }
}

}  // namespace
}  // namespace chorus

using namespace chorus;

extern "C" {

int32_t chorus_ln_modulate(const float* x, uint16_t* out, int64_t L, int32_t D, const float* mul0, const float* mul1,
                           const float* add0, const float* add1, int32_t plus_one, void* stream) {
  if (L < 0 || D <= 0) return CHORUS_E_ARG;
  if (L == 0) return CHORUS_OK;
  if (!x || !out || !mul0 || !add0) return CHORUS_E_ARG;
  if (D % 4) return CHORUS_E_SHAPE;
  if (!aligned16(x) || !aligned16(out) || !aligned16(mul0) || !aligned16(add0) || !aligned16(mul1) || !aligned16(add1))
    return CHORUS_E_ARG;
  hipStream_t s = (hipStream_t)stream;
  dim3 grid((unsigned)((L + 3) / 4)), block(256);
  float base = plus_one ? 1.0f : 0.0f;
  const size_t tab_bytes = (size_t)2 * D * sizeof(float);
  if (tab_bytes > 64 * 1024) return CHORUS_E_SHAPE;
#define LAUNCH_LN(NV) \
  hipLaunchKernelGGL((ln_modulate_kernel<NV>), grid, block, tab_bytes, s, x, out, (long)L, D, mul0, mul1, add0, add1, base)
  if (D == 256) LAUNCH_LN(1);
  else if (D == 1536) LAUNCH_LN(6);
  else if (D == 5120) LAUNCH_LN(20);
  else LAUNCH_LN(0);
#undef LAUNCH_LN
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

int32_t chorus_qk_norm_rope(const uint16_t* in, int64_t ld, const float* gain, uint16_t* out, int64_t L, int64_t Lpad,
                            int32_t H, int32_t dh, const int32_t* token_idx, int32_t gT, int32_t gH, int32_t gW,
                            int32_t rope, float out_scale, void* stream) {
  (void)gT;
  if (L < 0 || Lpad < L || H <= 0 || dh <= 0 || !(out_scale > 0.f) || !(out_scale < INFINITY)) return CHORUS_E_ARG;
  if (Lpad == 0) return CHORUS_OK;
  if (!in || !gain || !out) return CHORUS_E_ARG;
  if (dh % 8 || dh > 128 || (dh / 6) * 6 > dh || ld % 8) return CHORUS_E_SHAPE;
  if (rope && (gH <= 0 || gW <= 0)) return CHORUS_E_ARG;
  if (!aligned16(in) || !aligned16(out) || !aligned16(gain)) return CHORUS_E_ARG;
  hipStream_t s = (hipStream_t)stream;
  const int D_ = H * dh;  // widths with a register-resident row: 512 elements per chunk round
  if (D_ == 1536) {
    hipLaunchKernelGGL(qk_norm_rope_kernel<3>, dim3((unsigned)((Lpad + 3) / 4)), dim3(256), 0, s, in, (long)ld, gain, out,
                     (long)L, (long)Lpad, H, dh, token_idx, gH, gW, rope, out_scale);
  } else if (D_ == 5120) {
    hipLaunchKernelGGL(qk_norm_rope_kernel<10>, dim3((unsigned)((Lpad + 3) / 4)), dim3(256), 0, s, in, (long)ld, gain, out,
                     (long)L, (long)Lpad, H, dh, token_idx, gH, gW, rope, out_scale);
  } else if (D_ == 512) {
    hipLaunchKernelGGL(qk_norm_rope_kernel<1>, dim3((unsigned)((Lpad + 3) / 4)), dim3(256), 0, s, in, (long)ld, gain, out,
                     (long)L, (long)Lpad, H, dh, token_idx, gH, gW, rope, out_scale);
  } else {
    hipLaunchKernelGGL(qk_norm_rope_kernel<0>, dim3((unsigned)((Lpad + 3) / 4)), dim3(256), 0, s, in, (long)ld, gain, out,
                     (long)L, (long)Lpad, H, dh, token_idx, gH, gW, rope, out_scale);
  }
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

int32_t chorus_v_transpose(const uint16_t* in, int64_t ld, uint16_t* out, int64_t L, int64_t Lpad, int32_t D,
                           void* stream) {
  if (L < 0 || Lpad < L || D <= 0) return CHORUS_E_ARG;
  if (Lpad == 0) return CHORUS_OK;
  if (!in || !out) return CHORUS_E_ARG;
  if (D % 64 || Lpad % 64 || ld % 8) return CHORUS_E_SHAPE;
  if (!aligned16(in) || !aligned16(out)) return CHORUS_E_ARG;
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(v_transpose_kernel, dim3((unsigned)(Lpad / 64), (unsigned)(D / 64)), dim3(256), 0, s, in, (long)ld,
                     out, (long)L, (long)Lpad);
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

}  // extern "C"
