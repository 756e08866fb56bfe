// bf16 MFMA GEMM with fused epilogues: C = epi(A W^T + bias), A [M,K], W [N,K],
// both K-contiguous, fp32 accumulation with v_mfma_f32_32x32x16_bf16.
//
// Workgroup = 4 waves, tile BM x BN x 64. Each k-step the A and W tiles go
// global -> registers -> LDS (rows padded to 72 elements so the 16-byte operand
// reads of 16 consecutive lanes fall in distinct banks) while the MFMAs of the
// previous tile run. A wave owns a WM x WN sub-tile as (WM/32) x (WN/32) 32x32
// accumulators. Lane l of a 32x32 accumulator holds column n = l%32 and rows
// m = 4*(l/32) + 8*j + i (register 4j+i).
#include "chorus_ops.h"
#include "common.h"

namespace chorus {
namespace {

constexpr int BK = 64;
constexpr int LS = BK + 8;  // LDS row stride in elements

__device__ __forceinline__ float gelu_tanh_fast(float x) {
  // 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u)),  u = sqrt(2/pi) (x + 0.044715 x^3)
  float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
  float e = __builtin_amdgcn_exp2f(-2.0f * 1.4426950408889634f * u);
  return x * __builtin_amdgcn_rcpf(1.0f + e);
}

struct EpiArgs {
  void* out;
  const float* bias;
  const float* gate0;
  const float* gate1;
  float scale;
};

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(256, 2) void gemm_bf16_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
                                                        long M, int N, int K, EpiArgs ep, int tiles_m, int tiles_n) {
  constexpr int WAVES_N = BN / WN;
  static_assert((BM / WM) * (BN / WN) == 4, "4 waves");
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_LD = BM * 8 / 256, B_LD = BN * 8 / 256;
  constexpr int GM = 8;  // row-tiles per group: concurrently resident tiles form GM x (32/GM) patches

  __shared__ __attribute__((aligned(16))) uint16_t sA[BM * LS];
  __shared__ __attribute__((aligned(16))) uint16_t sB[BN * LS];

  const int ntiles = tiles_m * tiles_n;
  const int tile = xcd_remap(blockIdx.x, ntiles);
  const int per_group = GM * tiles_n;
  const int group = tile / per_group;
  const int first_m = group * GM;
  const int gsz = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
  const int in_group = tile - group * per_group;
  const int tm_idx = first_m + in_group % gsz;
  const int tn_idx = in_group / gsz;
  const long m0 = (long)tm_idx * BM;
  const int n0 = tn_idx * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int lrow = lane & 31, lk = (lane >> 5) * 8;

  // per-thread load slots: slot i covers tile row (tid>>3) + 32 i, 16-byte chunk tid&7;
  // rows past the end of the matrix are clamped (their products are never stored)
  const int lrow0 = tid >> 3, lch = (tid & 7) * 8;
  uint32_t aoff[A_LD], boff[B_LD];
  const uint16_t* Abase = A + m0 * (long)K + lch;
  const uint16_t* Bbase = W + (long)n0 * K + lch;
#pragma unroll
  for (int i = 0; i < A_LD; ++i) {
    long r = lrow0 + 32 * i;
    if (m0 + r > M - 1) r = M - 1 - m0;
    aoff[i] = (uint32_t)(r * K);
  }
#pragma unroll
  for (int i = 0; i < B_LD; ++i) {
    int r = lrow0 + 32 * i;
    if (n0 + r > N - 1) r = N - 1 - n0;
    boff[i] = (uint32_t)((long)r * K);
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  u32x4 ra[A_LD], rb[B_LD];
#pragma unroll
  for (int i = 0; i < A_LD; ++i) ra[i] = *reinterpret_cast<const u32x4*>(Abase + aoff[i]);
#pragma unroll
  for (int i = 0; i < B_LD; ++i) rb[i] = *reinterpret_cast<const u32x4*>(Bbase + boff[i]);

  const int KT = K / BK;
  for (int kt = 0; kt < KT; ++kt) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
      *reinterpret_cast<u32x4*>(&sA[(lrow0 + 32 * i) * LS + lch]) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
      *reinterpret_cast<u32x4*>(&sB[(lrow0 + 32 * i) * LS + lch]) = rb[i];
    }
    __syncthreads();
    if (kt + 1 < KT) {
#pragma unroll
      for (int i = 0; i < A_LD; ++i) ra[i] = *reinterpret_cast<const u32x4*>(Abase + (kt + 1) * BK + aoff[i]);
#pragma unroll
      for (int i = 0; i < B_LD; ++i) rb[i] = *reinterpret_cast<const u32x4*>(Bbase + (kt + 1) * BK + boff[i]);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = *reinterpret_cast<const bf16x8*>(&sA[(wm * WM + i * 32 + lrow) * LS + ks * 16 + lk]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        bfr[j] = *reinterpret_cast<const bf16x8*>(&sB[(wn * WN + j * 32 + lrow) * LS + ks * 16 + lk]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
  }

  // epilogue
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = n0 + wn * WN + j * 32 + lrow;
    if (n >= N) continue;
    const float bias = ep.bias ? ep.bias[n] : 0.f;
    float g = 1.f;
    if (EPI == CHORUS_EPI_RESID) {
      if (ep.gate0 || ep.gate1) g = (ep.gate0 ? ep.gate0[n] : 0.f) + (ep.gate1 ? ep.gate1[n] : 0.f);
      g *= ep.scale;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const long m = m0 + wm * WM + i * 32 + (lane >> 5) * 4 + 8 * (r >> 2) + (r & 3);
        if (m >= M) continue;
        float v = acc[i][j][r] + bias;
        if (EPI == CHORUS_EPI_BF16) {
          reinterpret_cast<uint16_t*>(ep.out)[m * N + n] = f32_to_bf16(v);
        } else if (EPI == CHORUS_EPI_GELU_BF16) {
          reinterpret_cast<uint16_t*>(ep.out)[m * N + n] = f32_to_bf16(gelu_tanh_fast(v));
        } else if (EPI == CHORUS_EPI_F32) {
          reinterpret_cast<float*>(ep.out)[m * N + n] = v;
        } else {
          float* o = reinterpret_cast<float*>(ep.out) + m * N + n;
          *o = *o + g * v;
        }
      }
    }
  }
}

template <int BM, int BN, int WM, int WN>
int32_t launch_gemm(const uint16_t* A, const uint16_t* W, long M, int N, int K, int epi, EpiArgs ep, hipStream_t s) {
  long tm = (M + BM - 1) / BM;
  int tn = (N + BN - 1) / BN;
  if (tm * tn > 0x7fffffffL) return CHORUS_E_SHAPE;
  dim3 grid((unsigned)(tm * tn)), block(256);
#define GEMM_LAUNCH(E) \
  hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WM, WN, E>), grid, block, 0, s, A, W, M, N, K, ep, (int)tm, tn)
  switch (epi) {
    case CHORUS_EPI_BF16: GEMM_LAUNCH(CHORUS_EPI_BF16); break;
    case CHORUS_EPI_GELU_BF16: GEMM_LAUNCH(CHORUS_EPI_GELU_BF16); break;
    case CHORUS_EPI_F32: GEMM_LAUNCH(CHORUS_EPI_F32); break;
    case CHORUS_EPI_RESID: GEMM_LAUNCH(CHORUS_EPI_RESID); break;
    default: return CHORUS_E_ARG;
  }
#undef GEMM_LAUNCH
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

}  // namespace
}  // namespace chorus

using namespace chorus;

extern "C" int32_t chorus_gemm_bf16(const uint16_t* A, const uint16_t* W, int64_t M, int32_t N, int32_t K,
                                    int32_t epilogue, void* out, const float* bias, const float* gate0,
                                    const float* gate1, float scale, void* stream) {
  if (M < 0 || N <= 0 || K <= 0) return CHORUS_E_ARG;
  if (M == 0) return CHORUS_OK;
  if (!A || !W || !out) return CHORUS_E_ARG;
  if (K % BK || N % 8) return CHORUS_E_SHAPE;
  if (!aligned16(A) || !aligned16(W) || !aligned16(out)) return CHORUS_E_ARG;
  EpiArgs ep{out, bias, gate0, gate1, scale};
  hipStream_t s = (hipStream_t)stream;
  // small problems get the smaller tile so that more workgroups exist
  long big_tiles = ((M + 255) / 256) * ((N + 127) / 128);
  if (big_tiles >= 256) return launch_gemm<256, 128, 128, 64>(A, W, (long)M, N, K, epilogue, ep, s);
  return launch_gemm<128, 64, 64, 32>(A, W, (long)M, N, K, epilogue, ep, s);
}
