// bf16 MFMA GEMM with fused epilogues: C = epi(A W^T + bias), A [M,K], W [N,K],
// both K-contiguous, fp32 accumulation with v_mfma_f32_32x32x16_bf16.
//
// Workgroup = 4 waves, tile BM x BN x 64. Each k-step the A and W tiles go
// global -> registers -> LDS (rows padded to 72 elements so the 16-byte operand
// reads of 16 consecutive lanes fall in distinct banks) while the MFMAs of the
// previous tile run. A wave owns a WM x WN sub-tile as (WM/32) x (WN/32) 32x32
// accumulators. The W fragment is the MFMA's row operand and the activation fragment its
// column operand, so lane l of a 32x32 accumulator holds ONE output row m = l%32 and the 16
// output columns n = 4*(l/32) + 8*g + e (register 4g+e): four consecutive columns per
// register group, which the epilogue moves as one 8-byte (bf16) or 16-byte (fp32) access.
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


// Epilogue for one lane: acc[i][j][4g+e] is C[m_i][n_j + 8g + e] with m_i = m_base + 32 i and
// n_j = n_base + 32 j (n_base already includes the lane's 4*(l/32)).
template <int EPI, int TM, int TN>
__device__ __forceinline__ void gemm_epilogue(const f32x16 (&acc)[TM][TN], const EpiArgs& ep, long m_base, int n_base,
                                              long M, int N) {
  if constexpr (EPI == CHORUS_EPI_RESID) {
    // Read-modify-write of the fp32 residual: all 4 * TM loads of a 32-column block are issued before the first store
    // (the compiler cannot hoist them itself: it must assume a store may alias a later load), so the block costs one
    // memory round trip instead of one per row group.
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int nj = n_base + 32 * j;
      f32x4 cur[4][TM];
      bool ok[4][TM];
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const long m = m_base + 32 * i;
          ok[g][i] = (nj + 8 * g < N) && (m < M);
          // unconditional loads from a clamped address (predicated ones end up in scratch)
          const long mc = m < M ? m : M - 1;
          const int nc = nj + 8 * g < N ? nj + 8 * g : 0;
          cur[g][i] = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(ep.out) + mc * N + nc);
        }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = nj + 8 * g;
        if (n >= N) continue;
        f32x4 bias = {0.f, 0.f, 0.f, 0.f};
        if (ep.bias) bias = *reinterpret_cast<const f32x4*>(ep.bias + n);
        f32x4 gate = {1.f, 1.f, 1.f, 1.f};
        if (ep.gate0 || ep.gate1) {
          gate = f32x4{0.f, 0.f, 0.f, 0.f};
          if (ep.gate0) gate += *reinterpret_cast<const f32x4*>(ep.gate0 + n);
          if (ep.gate1) gate += *reinterpret_cast<const f32x4*>(ep.gate1 + n);
        }
        gate *= ep.scale;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          if (!ok[g][i]) continue;
          const long m = m_base + 32 * i;
          f32x4 v = {acc[i][j][4 * g + 0], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
          *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(ep.out) + m * N + n) = cur[g][i] + gate * (v + bias);
        }
      }
    }
    return;
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int n = n_base + 32 * j + 8 * g;
      if (n >= N) continue;  // N % 8 == 0 and n % 4 == 0: the four columns are in or out together
      float4 bias = make_float4(0.f, 0.f, 0.f, 0.f);
      if (ep.bias) bias = *reinterpret_cast<const float4*>(ep.bias + n);
      float4 gate = make_float4(1.f, 1.f, 1.f, 1.f);
      if (EPI == CHORUS_EPI_RESID) {
        if (ep.gate0 || ep.gate1) {
          gate = make_float4(0.f, 0.f, 0.f, 0.f);
          if (ep.gate0) {
            float4 t = *reinterpret_cast<const float4*>(ep.gate0 + n);
            gate.x += t.x; gate.y += t.y; gate.z += t.z; gate.w += t.w;
          }
          if (ep.gate1) {
            float4 t = *reinterpret_cast<const float4*>(ep.gate1 + n);
            gate.x += t.x; gate.y += t.y; gate.z += t.z; gate.w += t.w;
          }
        }
        gate.x *= ep.scale; gate.y *= ep.scale; gate.z *= ep.scale; gate.w *= ep.scale;
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const long m = m_base + 32 * i;
        if (m >= M) continue;
        float v0 = acc[i][j][4 * g + 0] + bias.x, v1 = acc[i][j][4 * g + 1] + bias.y;
        float v2 = acc[i][j][4 * g + 2] + bias.z, v3 = acc[i][j][4 * g + 3] + bias.w;
        if (EPI == CHORUS_EPI_BF16 || EPI == CHORUS_EPI_GELU_BF16) {
          if (EPI == CHORUS_EPI_GELU_BF16) {
            v0 = gelu_tanh_fast(v0); v1 = gelu_tanh_fast(v1); v2 = gelu_tanh_fast(v2); v3 = gelu_tanh_fast(v3);
          }
          uint2 w;
          w.x = pack_bf16x2(v0, v1);
          w.y = pack_bf16x2(v2, v3);
          *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(ep.out) + m * N + n) = w;
        } else if (EPI == CHORUS_EPI_F32) {
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(ep.out) + m * N + n) = make_float4(v0, v1, v2, v3);
        } else {
          float4* o = reinterpret_cast<float4*>(reinterpret_cast<float*>(ep.out) + m * N + n);
          float4 c = *o;
          c.x += gate.x * v0; c.y += gate.y * v1; c.z += gate.z * v2; c.w += gate.w * v3;
          *o = c;
        }
      }
    }
  }
}

// bf16 epilogue through LDS: the wave's 128 x 64 tile is converted (bias, optional GELU) and
// written to a private LDS region as [m][n] in two halves of 64 rows, then read back with
// 8 lanes per row of 128 bytes, so every global store instruction writes 8 full 128-byte
// lines instead of 32 scattered 8-byte pieces. `cw` is this wave's region of 64 x 68 elements;
// the caller guarantees that no wave still reads the main-loop LDS it overlays.
constexpr int EPI_LDS_STRIDE = 64 + 4;
constexpr int EPI_LDS_WAVE = 64 * EPI_LDS_STRIDE;  // elements per wave

template <int EPI>
__device__ __forceinline__ void gemm_epilogue_bf16_lds(const f32x16 (&acc)[4][2], const EpiArgs& ep, uint16_t* cw,
                                                       long m_wave0, int n_wave0, long M, int N, int lane) {
  const int lrow = lane & 31, c4 = (lane >> 5) * 4;
  const int rrow = lane >> 3, rch = (lane & 7) * 8;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int nl = 32 * j + 8 * g + c4;  // column inside the wave tile
        const int n = n_wave0 + nl;
        float4 bias = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ep.bias && n < N) bias = *reinterpret_cast<const float4*>(ep.bias + n);
#pragma unroll
        for (int i2 = 0; i2 < 2; ++i2) {
          const f32x16& a = acc[2 * half + i2][j];
          float v0 = a[4 * g + 0] + bias.x, v1 = a[4 * g + 1] + bias.y, v2 = a[4 * g + 2] + bias.z,
                v3 = a[4 * g + 3] + bias.w;
          if (EPI == CHORUS_EPI_GELU_BF16) {
            v0 = gelu_tanh_fast(v0); v1 = gelu_tanh_fast(v1); v2 = gelu_tanh_fast(v2); v3 = gelu_tanh_fast(v3);
          }
          uint2 w;
          w.x = pack_bf16x2(v0, v1);
          w.y = pack_bf16x2(v2, v3);
          *reinterpret_cast<uint2*>(cw + (32 * i2 + lrow) * EPI_LDS_STRIDE + nl) = w;
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");  // LDS ops of one wave stay in order
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int row = 8 * it + rrow;
      const long m = m_wave0 + 64 * half + row;
      const int n = n_wave0 + rch;
      const u32x4 v = *reinterpret_cast<const u32x4*>(cw + row * EPI_LDS_STRIDE + rch);
      if (m < M && n < N) *reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(ep.out) + m * N + n) = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
  }
}

// fp32 residual epilogue through LDS for a 128 x 64 wave tile: 32 rows at a time are written to a private LDS
// region as [32][64] floats (row stride 68 floats, so the 16-byte writes of 16 lanes fall in distinct banks), then
// read back with 16 lanes per row, so every global load / store instruction moves four full 256-byte row segments
// of the residual instead of 32-byte pieces of 32 rows. `cw` is this wave's region of 32 x 68 floats; the caller
// guarantees that no wave still reads the main-loop LDS it overlays.
constexpr int EPI_F32_STRIDE = 64 + 4;
constexpr int EPI_F32_WAVE = 32 * EPI_F32_STRIDE;  // floats per wave

__device__ __forceinline__ void gemm_epilogue_resid_lds(const f32x16 (&acc)[4][2], const EpiArgs& ep, float* cw, long m_wave0,
                                                        int n_wave0, long M, int N, int lane) {
  const int lrow = lane & 31, c4 = (lane >> 5) * 4;
  const int rrow = lane >> 4, rcol = (lane & 15) * 4;  // read-back: 4 rows per instruction, 16 lanes per row
  const int n = n_wave0 + rcol;
  const bool n_ok = n < N;  // N % 8 == 0: the four columns are in or out together
  f32x4 bias = {0.f, 0.f, 0.f, 0.f}, gate = {1.f, 1.f, 1.f, 1.f};
  if (n_ok) {
    if (ep.bias) bias = *reinterpret_cast<const f32x4*>(ep.bias + n);
    if (ep.gate0 || ep.gate1) {
      gate = f32x4{0.f, 0.f, 0.f, 0.f};
      if (ep.gate0) gate += *reinterpret_cast<const f32x4*>(ep.gate0 + n);
      if (ep.gate1) gate += *reinterpret_cast<const f32x4*>(ep.gate1 + n);
    }
    gate *= ep.scale;
  }
  float* out = reinterpret_cast<float*>(ep.out);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    // the residual rows of this pass are requested before the LDS round trip
    f32x4 cur[8];
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      long m = m_wave0 + 32 * i + 4 * it + rrow;
      if (m > M - 1) m = M - 1;  // rows past the end read the last row (never stored)
      cur[it] = *reinterpret_cast<const f32x4*>(out + m * N + (n_ok ? n : 0));
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 v = {acc[i][j][4 * g + 0], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        *reinterpret_cast<f32x4*>(cw + lrow * EPI_F32_STRIDE + 32 * j + 8 * g + c4) = v;
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");  // LDS ops of one wave stay in order
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(cw + (4 * it + rrow) * EPI_F32_STRIDE + rcol);
      const long m = m_wave0 + 32 * i + 4 * it + rrow;
      if (n_ok && m < M) *reinterpret_cast<f32x4*>(out + m * N + n) = cur[it] + gate * (v + bias);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_sched_barrier(0);
  }
}

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
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    }
  }

  if constexpr (EPI == CHORUS_EPI_RESID && TM == 4 && TN == 2 && BM * LS * 2 >= 4 * EPI_F32_WAVE * 4) {
    __syncthreads();  // the staging regions overlay the A tile
    gemm_epilogue_resid_lds(acc, ep, reinterpret_cast<float*>(sA) + wave * EPI_F32_WAVE, m0 + wm * WM, n0 + wn * WN, M, N, lane);
  } else {
    gemm_epilogue<EPI, TM, TN>(acc, ep, m0 + wm * WM + lrow, n0 + wn * WN + (lane >> 5) * 4, M, N);
  }
}

// ---------------------------------------------------------------------------
// Large-problem kernel: 256 x 256 x 64 tiles, 8 waves (2 x 4, each 128 x 64), operands
// streamed global -> LDS directly (global_load_lds_dwordx4, no register staging, no
// LDS store instructions), two LDS stages, one barrier per k-step: after the barrier
// that publishes tile kt, the loads of tile kt+1 are issued into the other stage and
// stay in flight during the 32 MFMAs per wave of tile kt.
//
// A direct load writes the 64 lanes' 16-byte pieces to consecutive LDS addresses,
// i.e. 8 unpadded rows of 128 bytes. Bank conflicts are avoided by an XOR swizzle
// instead of padding: the 16-byte chunk c of row r lives at chunk position
// c ^ ((r >> 1) & 7); the loading lane for position p of row r fetches global chunk
// p ^ ((r >> 1) & 7). Sixteen consecutive rows read at one logical chunk then cover
// all 64 banks exactly once.
// ---------------------------------------------------------------------------
template <int EPI>
__global__ __launch_bounds__(512, 2) void gemm_dl_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
                                                         long M, int N, int K, EpiArgs ep, int tiles_m, int tiles_n) {
  constexpr int BM = 256, BN = 256, WM = 128, WN = 64;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int GM = 8;
  constexpr int STAGE = (BM + BN) * BK;  // elements per stage
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem_raw[];
  uint16_t* smem = reinterpret_cast<uint16_t*>(smem_raw);

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
  const int wm = wave >> 2, wn = wave & 3;
  const int lrow = lane & 31;

  // ---- loader: wave w, slot i covers tile rows 8*(4w+i) .. +8 of A and of W; lane -> (row, position)
  const int lr = lane >> 3, lp = lane & 7;
  const uint16_t* ga[4];
  const uint16_t* gb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = 8 * (4 * wave + i) + lr;           // row inside the 256-row tile
    const int ch = lp ^ ((r >> 1) & 7);              // global chunk that belongs at position lp
    long ra = m0 + r;
    if (ra > M - 1) ra = M - 1;
    int rb = n0 + r;
    if (rb > N - 1) rb = N - 1;
    ga[i] = A + ra * (long)K + ch * 8;
    gb[i] = W + (long)rb * K + ch * 8;
  }
  auto issue = [&](int kt, int stage) {
    uint16_t* sa = smem + stage * STAGE;
    uint16_t* sb = sa + BM * BK;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int rows0 = 8 * (4 * wave + i);
      __builtin_amdgcn_global_load_lds(ga[i] + (long)kt * BK, sa + rows0 * BK, 16, 0, 0);
      __builtin_amdgcn_global_load_lds(gb[i] + (long)kt * BK, sb + rows0 * BK, 16, 0, 0);
    }
  };

  // ---- operand read offsets (elements): row base + swizzled chunk for each k-substep
  const int sw = (lrow >> 1) & 7;
  int koff[BK / 16];
#pragma unroll
  for (int ks = 0; ks < BK / 16; ++ks) koff[ks] = ((2 * ks + (lane >> 5)) ^ sw) * 8;
  const int a_row0 = (wm * WM + lrow) * BK;
  const int b_row0 = BM * BK + (wn * WN + lrow) * BK;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int KTN = K / BK;
  issue(0, 0);
  for (int kt = 0; kt < KTN; ++kt) {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's pieces of tile kt are in LDS
    lds_barrier();                       // ... and everybody's; all waves are done with the other stage
    __builtin_amdgcn_sched_barrier(0);
    issue(kt + 1 < KTN ? kt + 1 : kt, (kt + 1) & 1);  // branch-free: the last step re-fetches its own tile into the idle stage
    const uint16_t* st = smem + (kt & 1) * STAGE;
    // Operand fragments are double-buffered in registers: the LDS reads of k-substep ks+1 are
    // issued ahead of the 8 MFMAs of substep ks, so a fragment is requested ~256 cycles before use.
    bf16x8 af[2][TM], bfr[2][TN];
    auto read_frags = [&](int ks, int set) {
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[set][j] = *reinterpret_cast<const bf16x8*>(st + b_row0 + j * 32 * BK + koff[ks]);
#pragma unroll
      for (int i = 0; i < TM; ++i) af[set][i] = *reinterpret_cast<const bf16x8*>(st + a_row0 + i * 32 * BK + koff[ks]);
    };
    read_frags(0, 0);
    __builtin_amdgcn_sched_group_barrier(0x020, 8, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      if (ks + 1 < BK / 16) read_frags(ks + 1, (ks + 1) & 1);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ks & 1][j], af[ks & 1][i], acc[i][j], 0, 0, 0);
      if (ks + 1 < BK / 16) __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);  // all reads of ks+1 first
      __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);                           // then the MFMAs of ks
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // drain the redundant last prefetch before the workgroup may exit

  if constexpr (EPI == CHORUS_EPI_BF16 || EPI == CHORUS_EPI_GELU_BF16) {
    lds_barrier();  // the staging regions overlay the operand stages
    gemm_epilogue_bf16_lds<EPI>(acc, ep, smem + wave * EPI_LDS_WAVE, m0 + wm * WM, n0 + wn * WN, M, N, lane);
  } else if constexpr (EPI == CHORUS_EPI_RESID) {
    lds_barrier();
    gemm_epilogue_resid_lds(acc, ep, reinterpret_cast<float*>(smem_raw) + wave * EPI_F32_WAVE, m0 + wm * WM, n0 + wn * WN, M, N,
                            lane);
  } else {
    gemm_epilogue<EPI, TM, TN>(acc, ep, m0 + wm * WM + lrow, n0 + wn * WN + (lane >> 5) * 4, M, N);
  }
}

int32_t launch_gemm_dl(const uint16_t* A, const uint16_t* W, long M, int N, int K, int epi, EpiArgs ep, hipStream_t s) {
  long tm = (M + 255) / 256;
  int tn = (N + 255) / 256;
  if (tm * tn > 0x7fffffffL) return CHORUS_E_SHAPE;
  dim3 grid((unsigned)(tm * tn)), block(512);
  const size_t smem = 2 * (256 + 256) * BK * sizeof(uint16_t);  // 128 KB
#define GEMM_DL(E)                                                                              \
  {                                                                                             \
    auto kern = gemm_dl_kernel<E>;                                                              \
    static DynLdsOnce once;                                                                     \
    CHK_STATUS(once.ensure(reinterpret_cast<const void*>(kern), (int)smem));                    \
    hipLaunchKernelGGL(kern, grid, block, smem, s, A, W, M, N, K, ep, (int)tm, tn);             \
  }
  switch (epi) {
    case CHORUS_EPI_BF16: GEMM_DL(CHORUS_EPI_BF16); break;
    case CHORUS_EPI_GELU_BF16: GEMM_DL(CHORUS_EPI_GELU_BF16); break;
    case CHORUS_EPI_F32: GEMM_DL(CHORUS_EPI_F32); break;
    case CHORUS_EPI_RESID: GEMM_DL(CHORUS_EPI_RESID); break;
    default: return CHORUS_E_ARG;
  }
#undef GEMM_DL
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
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

extern "C" int32_t chorus_gemm_bf16_kernel(const uint16_t* A, const uint16_t* W, int64_t M, int32_t N, int32_t K,
                                           int32_t epilogue, void* out, const float* bias, const float* gate0,
                                           const float* gate1, float scale, int32_t kernel, void* stream) {
  if (M < 0 || N <= 0 || K <= 0) return CHORUS_E_ARG;
  if (kernel < 0 || kernel > 3) return CHORUS_E_ARG;
  if (M == 0) return CHORUS_OK;
  if (!A || !W || !out) return CHORUS_E_ARG;
  if (K % BK || N % 8) return CHORUS_E_SHAPE;
  if (!aligned16(A) || !aligned16(W) || !aligned16(out) || !aligned16(bias) || !aligned16(gate0) || !aligned16(gate1))
    return CHORUS_E_ARG;
  EpiArgs ep{out, bias, gate0, gate1, scale};
  hipStream_t s = (hipStream_t)stream;
  if (kernel == 1) return launch_gemm<128, 64, 64, 32>(A, W, (long)M, N, K, epilogue, ep, s);
  if (kernel == 2) return launch_gemm<256, 128, 128, 64>(A, W, (long)M, N, K, epilogue, ep, s);
  if (kernel == 3) return launch_gemm_dl(A, W, (long)M, N, K, epilogue, ep, s);
  // small problems get the smaller tile so that more workgroups exist; between the two large tiles the choice goes
  // by rounds of 256 workgroups: a 256 x 128 tile takes about 0.6 of the time of a 256 x 256 one
  long big_tiles = ((M + 255) / 256) * ((N + 127) / 128);
  long dl_tiles = ((M + 255) / 256) * ((N + 255) / 256);
  if (dl_tiles >= 256) {
    const double t_dl = (double)((dl_tiles + 255) / 256);
    const double t_big = 0.6 * (double)((big_tiles + 255) / 256);
    if (t_dl <= t_big) return launch_gemm_dl(A, W, (long)M, N, K, epilogue, ep, s);
  }
  if (big_tiles >= 256) return launch_gemm<256, 128, 128, 64>(A, W, (long)M, N, K, epilogue, ep, s);
  return launch_gemm<128, 64, 64, 32>(A, W, (long)M, N, K, epilogue, ep, s);
}

extern "C" int32_t chorus_gemm_bf16(const uint16_t* A, const uint16_t* W, int64_t M, int32_t N, int32_t K,
                                    int32_t epilogue, void* out, const float* bias, const float* gate0,
                                    const float* gate1, float scale, void* stream) {
  return chorus_gemm_bf16_kernel(A, W, M, N, K, epilogue, out, bias, gate0, gate1, scale, 0, stream);
}
