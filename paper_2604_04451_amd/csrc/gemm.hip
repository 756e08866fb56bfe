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
  // 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u)),  u = sqrt(2/pi) (x + 0.044715 x^3); the exponent is taken in base 2:
  // -2u log2(e) = -x (2.3022082 + 0.10294324 x^2)
  const float t = x * x;
  const float p = __builtin_fmaf(t, -0.10294324f, -2.3022082f);
  const float e = __builtin_amdgcn_exp2f(p * x);
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
// Large-problem kernel: 256 x 256 x 64 tiles, four waves (one per SIMD), each wave a 128 x 128 quadrant as 8 x 8
// accumulators of v_mfma_f32_16x16x32_bf16 (256 accumulator registers). Per unit of work a 16x16x32 MFMA reads and
// writes half the accumulator registers of a 32x32x16 one (k = 32 per instruction instead of 16), which is what the
// power-managed part rewards; a 16-byte LDS fragment (16 rows x 8 k per quarter wave) feeds eight MFMAs.
//
// Both operands stream global -> LDS directly (global_load_lds_dwordx4: no register staging, no LDS store
// instructions) into two 64 KB stages. A direct load writes the 64 lanes' 16-byte pieces to consecutive LDS
// addresses, i.e. 8 unpadded rows of 128 bytes. Bank conflicts are avoided by an XOR swizzle instead of padding: the
// 16-byte chunk c of row r lives at chunk position c ^ ((r >> 1) & 7); the loading lane for position p of row r
// fetches global chunk p ^ ((r >> 1) & 7). (A 16-byte-per-lane LDS read is served 16 lanes a cycle: the four-lane
// groups of one half wave whose group index has the same bit parity, groups 0, 3, 5, 6 together and 1, 2, 4, 7. With
// lane = 16 * chunk + row those are rows 0-3 and 12-15 of one chunk with rows 4-11 of its neighbour, which this
// swizzle spreads over all 64 banks: measured, no conflict cycles.)
//
// Operand layout of v_mfma_f32_16x16x32_bf16: lane l supplies row (or column) l % 16 and the 8 k-values
// 8 (l / 16) .. + 8; it receives column l % 16 and rows 4 (l / 16) .. + 4 of the 16 x 16 result. The weight fragment is
// the row operand and the activation fragment the column operand, so a lane holds one output row m and four
// consecutive output columns n.
//
// One loop iteration per k-step, hand-laid for a single wave per SIMD (nothing else hides a gap between two MFMAs):
// half-step 0 (64 MFMAs) with the LDS reads of half-step 1's fragments; vmcnt(0) + barrier; half-step 1 (64 MFMAs) with
// the LDS reads of the next step's first fragments and the 16 loads of the step after next (their stage is free behind
// the barrier). Every read and load stands alone between two MFMAs.
// The MFMAs are volatile assembly, in place on their accumulators: left to the register allocator every result gets
// a new home, at the price of several hundred accumulator moves per k-step.
// ---------------------------------------------------------------------------

// WB = 16 x 16 blocks along each side of a wave's quadrant: 8 (256 x 256 tiles) or 4 (128 x 128 tiles).
//
// bf16 (optionally GELU) epilogue of the 16x16 layout: 32 output rows at a time go through a private LDS region as
// [32][16 WB] bf16 (row stride 16 WB + 8), then leave as full row segments of the quadrant (256 or 128 bytes).
template <int WB> constexpr int e16_bf_stride() { return 16 * WB + 8; }
template <int WB> constexpr int e16_bf_wave() { return 32 * e16_bf_stride<WB>(); }  // elements per wave
template <int EPI, int WB>
__device__ __forceinline__ void gemm16_epilogue_bf16(const f32x4 (&acc)[8][8], const EpiArgs& ep, uint16_t* cw, long m_wave0,
                                                     int n_wave0, long M, int N, int lane) {
  constexpr int E16_BF_STRIDE = e16_bf_stride<WB>();
  constexpr int LPR = 2 * WB, RPI = 64 / LPR;  // read-back: LPR lanes x 16 bytes per row, RPI rows per instruction
  const int lj = lane & 15, lg = lane >> 4;
  const int rrow = lane / LPR, rcol = (lane % LPR) * 8;
  float4 bias[WB];
#pragma unroll
  for (int nb = 0; nb < WB; ++nb) {
    const int n = n_wave0 + 16 * nb + 4 * lg;
    bias[nb] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (ep.bias && n < N) bias[nb] = *reinterpret_cast<const float4*>(ep.bias + n);
  }
#pragma unroll
  for (int mp = 0; mp < WB / 2; ++mp) {  // pairs of 16-row blocks
#pragma unroll
    for (int mh = 0; mh < 2; ++mh)
#pragma unroll
      for (int nb = 0; nb < WB; ++nb) {
        const f32x4& a = acc[nb][2 * mp + mh];
        float v0 = a[0] + bias[nb].x, v1 = a[1] + bias[nb].y, v2 = a[2] + bias[nb].z, v3 = a[3] + bias[nb].w;
        if (EPI == CHORUS_EPI_GELU_BF16) {
          v0 = gelu_tanh_fast(v0); v1 = gelu_tanh_fast(v1); v2 = gelu_tanh_fast(v2); v3 = gelu_tanh_fast(v3);
        }
        uint2 w;
        w.x = pack_bf16x2(v0, v1);
        w.y = pack_bf16x2(v2, v3);
        *reinterpret_cast<uint2*>(cw + (16 * mh + lj) * E16_BF_STRIDE + 16 * nb + 4 * lg) = w;
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
#pragma unroll
    for (int it = 0; it < 32 / RPI; ++it) {
      const int row = RPI * it + rrow;
      const long m = m_wave0 + 32 * mp + row;
      const int n = n_wave0 + rcol;
      const u32x4 v = *reinterpret_cast<const u32x4*>(cw + row * E16_BF_STRIDE + rcol);
      // streaming store: an output tile is not read again by this kernel, and left to the default policy the written
      // lines push the operand panels that the next tiles share out of the L2 (measured: 14-19 % on the widest output)
      if (m < M && n < N) __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(reinterpret_cast<uint16_t*>(ep.out) + m * N + n));
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_sched_barrier(0);
  }
}

// fp32 gated-residual epilogue of the 16x16 layout: 16 output rows at a time through a private LDS region as
// [16][16 WB] fp32 (row stride 16 WB + 4), read back with 4 WB lanes per row; the residual rows are requested before the
// LDS round trip. out[m][n] += gate[n] * scale * (acc + bias[n]).
template <int WB> constexpr int e16_f32_stride() { return 16 * WB + 4; }
template <int WB> constexpr int e16_f32_wave() { return 16 * e16_f32_stride<WB>(); }  // floats per wave
template <int WB>
__device__ __forceinline__ void gemm16_epilogue_resid(const f32x4 (&acc)[8][8], const EpiArgs& ep, float* cw, long m_wave0,
                                                      int n_wave0, long M, int N, int lane) {
  constexpr int E16_F32_STRIDE = e16_f32_stride<WB>();
  constexpr int LPR = 4 * WB, RPI = 64 / LPR;  // read-back: LPR lanes x 16 bytes per row, RPI rows per instruction
  const int lj = lane & 15, lg = lane >> 4;
  const int rrow = lane / LPR, rcol = (lane % LPR) * 4;
  const int n = n_wave0 + rcol;
  const bool n_ok = n < N;
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
  // The residual rows of block mb + 1 are requested before the results of block mb are stored: memory operations
  // retire in order, so a load issued behind a block's stores could only be consumed once those stores had drained.
  f32x4 cur[2][WB];
  auto fetch = [&](int mb, f32x4 (&dst)[WB]) {
#pragma unroll
    for (int it = 0; it < WB; ++it) {
      long m = m_wave0 + 16 * mb + RPI * it + rrow;
      if (m > M - 1) m = M - 1;  // rows past the end read the last row (never stored)
      dst[it] = *reinterpret_cast<const f32x4*>(out + m * N + (n_ok ? n : 0));
    }
  };
  fetch(0, cur[0]);
#pragma unroll
  for (int mb = 0; mb < WB; ++mb) {
#pragma unroll
    for (int nb = 0; nb < WB; ++nb) *reinterpret_cast<f32x4*>(cw + lj * E16_F32_STRIDE + 16 * nb + 4 * lg) = acc[nb][mb];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    if (mb + 1 < WB) fetch(mb + 1, cur[(mb + 1) & 1]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int it = 0; it < WB; ++it) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(cw + (RPI * it + rrow) * E16_F32_STRIDE + rcol);
      const long m = m_wave0 + 16 * mb + RPI * it + rrow;
      if (n_ok && m < M) *reinterpret_cast<f32x4*>(out + m * N + n) = cur[mb & 1][it] + gate * (v + bias);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Epilogue of the 4-wave 16x16 kernels: wave (wm, wn) holds rows m0 + 16 WB wm .. + 16 WB, columns n0 + 16 WB wn .. + 16 WB.
template <int EPI, int WB>
__device__ __forceinline__ void gemm16_finish(f32x4 (&acc)[8][8], const EpiArgs& ep, uint8_t* smem_raw, int wave, int wm, int wn,
                                              long m0, int n0, long M, int N, int lane) {
  constexpr int WT = 16 * WB;  // rows and columns of a wave's quadrant
  uint16_t* smem = reinterpret_cast<uint16_t*>(smem_raw);
  const int lj = lane & 15, lg = lane >> 4;
  if constexpr (EPI == CHORUS_EPI_BF16 || EPI == CHORUS_EPI_GELU_BF16) {
    gemm16_epilogue_bf16<EPI, WB>(acc, ep, smem + wave * e16_bf_wave<WB>(), m0 + wm * WT, n0 + wn * WT, M, N, lane);
  } else if constexpr (EPI == CHORUS_EPI_RESID) {
    gemm16_epilogue_resid<WB>(acc, ep, reinterpret_cast<float*>(smem_raw) + wave * e16_f32_wave<WB>(), m0 + wm * WT, n0 + wn * WT, M,
                              N, lane);
  } else {
    // plain fp32: a lane stores its four consecutive columns of every block
#pragma unroll
    for (int nb = 0; nb < WB; ++nb) {
      const int n = n0 + wn * WT + 16 * nb + 4 * lg;
      if (n >= N) continue;
      f32x4 bias = {0.f, 0.f, 0.f, 0.f};
      if (ep.bias) bias = *reinterpret_cast<const f32x4*>(ep.bias + n);
#pragma unroll
      for (int mb = 0; mb < WB; ++mb) {
        const long m = m0 + wm * WT + 16 * mb + lj;
        if (m < M) *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(ep.out) + m * N + n) = acc[nb][mb] + bias;
      }
    }
  }
}

template <int EPI, int WB>
__global__ __launch_bounds__(256, 1) void gemm_w16_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ W,
                                                          long M, int N, int K, EpiArgs ep, int tiles_m, int tiles_n) {
  static_assert(WB == 8 || WB == 4, "quadrants of 8 x 8 or 4 x 4 blocks");
  constexpr int BM = 32 * WB, BN = 32 * WB;
  constexpr int WT = 16 * WB;  // rows and columns of a wave's quadrant
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
  // Within a group the tiles that run together on one XCD share operands in its L2. Normally they are taken row tile
  // fastest (8 row tiles x 4 column tiles at a time). When the activation rows are long and the weight matrix is only
  // a few tiles wide, column tile fastest is better: all column tiles of a row tile run together, so every activation
  // panel, the operand too big for any cache, leaves HBM once.
  const bool n_fastest = tiles_n <= 8 && K >= 4096;
  const int tm_idx = n_fastest ? first_m + in_group / tiles_n : first_m + in_group % gsz;
  const int tn_idx = n_fastest ? in_group % tiles_n : in_group / gsz;
  const long m0 = (long)tm_idx * BM;
  const int n0 = tn_idx * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int lj = lane & 15, lg = lane >> 4;

  // ---- loader: wave w, slot i (0..WB-1) covers tile rows 8*(WB w+i) .. +8 of A and of W; lane -> (row, position)
  const int lr = lane >> 3, lp = lane & 7;
  // (the arrays that the lambdas below capture have the large tile's size for either tile: a bound that depends on
  // the template parameter loses the kernel's host-side stub)
  const uint16_t* ga[8];
  const uint16_t* gb[8];
#pragma unroll
  for (int i = 0; i < WB; ++i) {
    const int r = 8 * (WB * wave + i) + lr;
    const int ch = lp ^ ((r >> 1) & 7);  // global chunk that belongs at position lp
    long ra = m0 + r;
    if (ra > M - 1) ra = M - 1;
    int rb = n0 + r;
    if (rb > N - 1) rb = N - 1;
    ga[i] = A + ra * (long)K + ch * 8;
    gb[i] = W + (long)rb * K + ch * 8;
  }
  auto issue = [&](int kt, int stage, int t0, int t1) {  // loads t0 .. t1-1 of the 2 WB per k-step (even: A rows, odd: W rows)
    uint16_t* sa = smem + stage * STAGE;
    uint16_t* sb = sa + BM * BK;
#pragma unroll
    for (int t = t0; t < t1; ++t) {
      const int i = t >> 1;
      const int rows0 = 8 * (WB * wave + i);
      if (t & 1)
        __builtin_amdgcn_global_load_lds(gb[i] + (long)kt * BK, sb + rows0 * BK, 16, 0, 0);
      else
        __builtin_amdgcn_global_load_lds(ga[i] + (long)kt * BK, sa + rows0 * BK, 16, 0, 0);
    }
  };

  // ---- fragment read offsets (elements): row l % 16 of a 16-row block, 16-byte chunk 4 h + l / 16, swizzled by the row
  const int sw = (lj >> 1) & 7;
  int koff[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) koff[h] = ((4 * h + lg) ^ sw) * 8;
  const int a_row0 = (wm * WT + lj) * BK;
  const int b_row0 = BM * BK + (wn * WT + lj) * BK;

  f32x4 acc[8][8];  // [n block][m block]; the WB x WB corner is used
#pragma unroll
  for (int nb = 0; nb < WB; ++nb)
#pragma unroll
    for (int mb = 0; mb < WB; ++mb) acc[nb][mb] = f32x4{0.f, 0.f, 0.f, 0.f};

  bf16x8 af[2][8], bfr[2][8];
  // fragment f of a half-step: 0 .. WB-1 the activation blocks (m), WB .. 2 WB-1 the weight blocks (n)
  auto read_frag = [&](const uint16_t* st, int h, int set, int f) {
    if (f < WB)
      af[set][f] = *reinterpret_cast<const bf16x8*>(st + a_row0 + f * 16 * BK + koff[h]);
    else
      bfr[set][f - WB] = *reinterpret_cast<const bf16x8*>(st + b_row0 + (f - WB) * 16 * BK + koff[h]);
  };
  // MFMAs g0 .. g1-1 of the WB * WB of a half-step, weight block major: g = WB nb + mb. In place on the accumulator
  // registers (left to itself the register allocator gives every result a new home and pays with hundreds of
  // accumulator moves per k-step); being volatile they also keep their place between the loads written around them.
  auto mfmas = [&](int set, int g0, int g1) {
#pragma unroll
    for (int g = g0; g < g1; ++g)
      asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[g / WB][g % WB]) : "v"(bfr[set][g / WB]), "v"(af[set][g % WB]));
  };
  // order in which the fragments of a half-step are fetched: what its first MFMAs need comes first (the first weight
  // block, the activation blocks, the other weight blocks)
  auto frag_order = [](int i) { return i == 0 ? WB : (i <= WB ? i - 1 : i); };

  // Schedule of one k-step (2 WB^2 MFMAs a wave in 4 WB slots of WB / 2: 128 MFMAs in 32 slots of four for the large
  // tile). The barrier sits between the two half-steps. In the
  // first half a wave fetches its fragments of the second half (same stage); at the barrier every wave holds all its
  // fragments of the current stage in registers and its own pieces of the next stage, requested a whole half-step
  // earlier, have landed. Behind it the stage just consumed is free: the second half issues the loads of the step after
  // next into it, one a slot, and fetches the next step's first-half fragments from the other stage. Fragment reads are
  // packed into the first kReadSlots slots of a half so that the last of them has returned when the half ends. With one
  // wave per SIMD nothing else feeds the matrix pipe while this wave issues something that is not an MFMA, so reads and
  // loads stand one at a time between single MFMAs, where they issue in the shadow of the MFMA in front of them, and
  // the wave index is kept in a scalar register so that the LDS address of a load costs no vector instruction.
  constexpr int NS = 2 * WB;              // slots of a half-step = fragments of a half-step = loads of a k-step
  constexpr int MPS = WB / 2;             // MFMAs of a slot
  constexpr int kReadSlots = 3 * WB / 2;  // 12 of 16 (6 of 8)
  const int KTN = K / BK;
  auto clampk = [&](int k) { return k < KTN ? k : KTN - 1; };  // past the end: re-fetch the last tile into an idle stage
  // reads of slot f: one fragment, two in the first NS - kReadSlots slots (which = 0: the first, 1: the second)
  auto read_of_slot = [&](const uint16_t* stg, int h, int set, int f, int which) {
    constexpr int kDouble = NS - kReadSlots;
    if (f < kDouble)
      read_frag(stg, h, set, frag_order(2 * f + which));
    else if (f < kReadSlots && which == 0)
      read_frag(stg, h, set, frag_order(f + kDouble));
  };
  issue(0, 0, 0, NS);
  issue(clampk(1), 1, 0, NS);
  // vmcnt(NS): the first step's pieces are in LDS, the second step's may be in flight
  if constexpr (WB == 8)
    __builtin_amdgcn_s_waitcnt(0x4F70);
  else
    __builtin_amdgcn_s_waitcnt(0x0F78);
  lds_barrier();
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int f = 0; f < NS; ++f) read_frag(smem, 0, 0, frag_order(f));
  __builtin_amdgcn_sched_barrier(0);

  for (int kt = 0; kt < KTN; ++kt) {
    const uint16_t* st = smem + (kt & 1) * STAGE;
    const uint16_t* stn = smem + ((kt + 1) & 1) * STAGE;
    const int k2 = clampk(kt + 2);
    // ---- half-step 0: WB^2 MFMAs and the fragment reads of half-step 1
#pragma unroll
    for (int f = 0; f < NS; ++f) {
      mfmas(0, MPS * f, MPS * f + 1);
      __builtin_amdgcn_sched_barrier(0);
      read_of_slot(st, 1, 1, f, 0);
      __builtin_amdgcn_sched_barrier(0);
      mfmas(0, MPS * f + 1, MPS * f + 2);
      __builtin_amdgcn_sched_barrier(0);
      read_of_slot(st, 1, 1, f, 1);
      __builtin_amdgcn_sched_barrier(0);
      mfmas(0, MPS * f + 2, MPS * f + MPS);
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's pieces of step kt+1 are in LDS
    lds_barrier();                       // every wave has all its fragments of this stage in registers
    __builtin_amdgcn_sched_barrier(0);
    // ---- half-step 1: WB^2 MFMAs, the next step's first-half fragments, the loads of step kt+2 into the stage just freed
#pragma unroll
    for (int f = 0; f < NS; ++f) {
      mfmas(1, MPS * f, MPS * f + 1);
      __builtin_amdgcn_sched_barrier(0);
      read_of_slot(stn, 0, 0, f, 0);
      __builtin_amdgcn_sched_barrier(0);
      mfmas(1, MPS * f + 1, MPS * f + 2);
      __builtin_amdgcn_sched_barrier(0);
      read_of_slot(stn, 0, 0, f, 1);
      __builtin_amdgcn_sched_barrier(0);
      mfmas(1, MPS * f + 2, MPS * f + MPS - 1);  // (none for the small tile)
      __builtin_amdgcn_sched_barrier(0);
      issue(k2, kt & 1, f, f + 1);
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (MPS > 2) mfmas(1, MPS * f + MPS - 1, MPS * f + MPS);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the look-ahead loads of the last step have landed
  // The compiler does not know the assembly above for MFMAs and so keeps no distance between the last of them and the
  // first instruction that reads an accumulator: cover the longest such distance explicitly. The wait is tied to the
  // accumulators of the last four MFMAs (operands of the statement), so that no copy or spill of one of them can be
  // placed in front of it; every other accumulator was written at least four MFMAs earlier.
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15"
               : "+a"(acc[WB - 1][WB - 1]), "+a"(acc[WB - 1][WB - 2]), "+a"(acc[WB - 1][WB - 3]), "+a"(acc[WB - 1][WB - 4]));
  lds_barrier();  // the staging regions of the epilogue overlay the operand stages
  gemm16_finish<EPI, WB>(acc, ep, smem_raw, wave, wm, wn, m0, n0, M, N, lane);
}

template <int WB>
int32_t launch_gemm_w16(const uint16_t* A, const uint16_t* W, long M, int N, int K, int epi, EpiArgs ep, hipStream_t s) {
  constexpr int T = 32 * WB;  // tile side: 256 or 128
  long tm = (M + T - 1) / T;
  int tn = (N + T - 1) / T;
  if (tm * tn > 0x7fffffffL) return CHORUS_E_SHAPE;
  dim3 grid((unsigned)(tm * tn)), block(256);
  const size_t smem = 2 * (T + T) * BK * sizeof(uint16_t);  // 128 KB (64 KB)
#define GEMM_W16(E)                                                                             \
  {                                                                                             \
    auto kern = gemm_w16_kernel<E, WB>;                                                         \
    static DynLdsOnce once;                                                                     \
    CHK_STATUS(once.ensure(reinterpret_cast<const void*>(kern), (int)smem));                    \
    hipLaunchKernelGGL(kern, grid, block, smem, s, A, W, M, N, K, ep, (int)tm, tn);             \
  }
  switch (epi) {
    case CHORUS_EPI_BF16: GEMM_W16(CHORUS_EPI_BF16); break;
    case CHORUS_EPI_GELU_BF16: GEMM_W16(CHORUS_EPI_GELU_BF16); break;
    case CHORUS_EPI_F32: GEMM_W16(CHORUS_EPI_F32); break;
    case CHORUS_EPI_RESID: GEMM_W16(CHORUS_EPI_RESID); break;
    default: return CHORUS_E_ARG;
  }
#undef GEMM_W16
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
  if (kernel < 0 || kernel > 4) return CHORUS_E_ARG;
  if (M == 0) return CHORUS_OK;
  if (!A || !W || !out) return CHORUS_E_ARG;
  if (K % BK || N % 8) return CHORUS_E_SHAPE;
  if (!aligned16(A) || !aligned16(W) || !aligned16(out) || !aligned16(bias) || !aligned16(gate0) || !aligned16(gate1))
    return CHORUS_E_ARG;
  EpiArgs ep{out, bias, gate0, gate1, scale};
  hipStream_t s = (hipStream_t)stream;
  if (kernel == 1) return launch_gemm<128, 64, 64, 32>(A, W, (long)M, N, K, epilogue, ep, s);
  if (kernel == 2) return launch_gemm<256, 128, 128, 64>(A, W, (long)M, N, K, epilogue, ep, s);
  if (kernel == 3) return launch_gemm_w16<8>(A, W, (long)M, N, K, epilogue, ep, s);
  if (kernel == 4) return launch_gemm_w16<4>(A, W, (long)M, N, K, epilogue, ep, s);
  // Automatic choice: the estimated time of each tile shape, in microseconds, from fits to measurements on this chip
  // at K = 1536 and K = 8960, M from 48 to 32760 and N = 1536, 4608 and 8960 (a constant for prologue and epilogue
  // plus a cost per element of K). The 256 x 256 and 256 x 128 tiles run one workgroup per compute unit, so they go in
  // rounds of 256 workgroups (the figures are those of a full round: a round that fills few units runs faster, and
  // there a smaller tile is chosen anyway). The 128 x 128 and 128 x 64 tiles keep several workgroups per unit in
  // flight, so their time grows with the tile count past the first 256.
  const double k = (double)K;
  const long tiles_n256 = (N + 255) / 256;
  const bool f32_out = epilogue == CHORUS_EPI_F32 || epilogue == CHORUS_EPI_RESID;
  auto t256 = [&](long m) { return (double)((((m + 255) / 256) * tiles_n256 + 255) / 256) * (2.0 + 0.0265 * k); };
  auto t128 = [&](long m) { return (double)((((m + 255) / 256) * ((N + 127) / 128) + 255) / 256) * (9.0 + 0.0177 * k); };
  auto t128sq = [&](long m) {  // two workgroups per unit: up to 256 tiles one each, then rounds of 512
    const long tiles = ((m + 127) / 128) * ((N + 127) / 128);
    const double one = (f32_out ? 6.0 : -2.0) + 0.0099 * k, round512 = (f32_out ? 9.0 : 1.0) + 0.0162 * k;
    if (tiles <= 256) return one;
    if (tiles <= 512) return one + (double)(tiles - 256) / 256.0 * (round512 - one);
    return (double)((tiles + 511) / 512) * round512;
  };
  auto t64 = [&](long m) {
    const long small_tiles = ((m + 127) / 128) * ((N + 63) / 64);
    return (5.6 + 0.0084 * k) + (small_tiles > 256 ? (double)(small_tiles - 256) / 256.0 * (0.8 + 0.0057 * k) : 0.0);
  };
  auto t_best = [&](long m) { return fmin(fmin(t256(m), t128(m)), fmin(t128sq(m), t64(m))); };
  auto launch_best = [&](const uint16_t* a, long m, const EpiArgs& e) {
    const double a256 = t256(m), a128 = t128(m), a128sq = t128sq(m), a64 = t64(m), best = t_best(m);
    if (a256 <= best) return launch_gemm_w16<8>(a, W, m, N, K, epilogue, e, s);
    if (a128sq <= best) return launch_gemm_w16<4>(a, W, m, N, K, epilogue, e, s);
    if (a128 <= a64) return launch_gemm<256, 128, 128, 64>(a, W, m, N, K, epilogue, e, s);
    return launch_gemm<128, 64, 64, 32>(a, W, m, N, K, epilogue, e, s);
  };
  // A last round of 256 x 256 tiles that fills a small part of the chip costs a whole round. The rows can be cut
  // instead: the row tiles that make up whole rounds go to the 256 x 256 kernel, the rows left over to whichever
  // kernel suits that many rows, in a second launch behind the first. Taken when the estimate is better by 5 %.
  const long tiles256 = ((M + 255) / 256) * tiles_n256;
  const long head_rows = tiles256 > 256 ? (tiles256 / 256 * 256 / tiles_n256) * 256 : 0;
  if (head_rows > 0 && head_rows < M) {
    const long rest = (long)M - head_rows;
    if (t256(head_rows) + t_best(rest) < 0.95 * t_best((long)M)) {
      const int32_t rc = launch_gemm_w16<8>(A, W, head_rows, N, K, epilogue, ep, s);
      if (rc != CHORUS_OK) return rc;
      const size_t out_elt = (epilogue == CHORUS_EPI_F32 || epilogue == CHORUS_EPI_RESID) ? 4 : 2;
      EpiArgs ep_rest = ep;
      ep_rest.out = static_cast<uint8_t*>(out) + (size_t)head_rows * (size_t)N * out_elt;
      return launch_best(A + (size_t)head_rows * (size_t)K, rest, ep_rest);
    }
  }
  return launch_best(A, (long)M, ep);
}

extern "C" int32_t chorus_gemm_bf16(const uint16_t* A, const uint16_t* W, int64_t M, int32_t N, int32_t K,
                                    int32_t epilogue, void* out, const float* bias, const float* gate0,
                                    const float* gate1, float scale, void* stream) {
  return chorus_gemm_bf16_kernel(A, W, M, N, K, epilogue, out, bias, gate0, gate1, scale, 0, stream);
}
