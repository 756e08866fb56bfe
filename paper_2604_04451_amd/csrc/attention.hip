// Flash-style attention for gfx950: O = softmax(g_j * (Q K^T) / sqrt(dh)) V, bf16
// operands on the matrix pipe, fp32 online softmax, logits never leave registers.
// Used for the block's 3-D self-attention (g = 1) and for the text cross-attention
// with TGAA key amplification (Eq. 2: scaling key j by gamma_k scales logit column j).
// Two kernels of one design: attention_pp_kernel on v_mfma_f32_32x32x16_bf16 (64-key
// tiles: key sequences shorter than 512 or padded to 64), described first, and
// attention_pp16_kernel on v_mfma_f32_16x16x32_bf16 (128-key tiles: self-attention and
// the text cross-attention from 512 keys on), whose differences are described in front of it.
// Both take the optional per-key logit factor.
//
// Work split: a workgroup of 8 waves owns 256 query rows of one head (32 per wave, held in
// registers) and sweeps all keys in tiles of 64 (128 in the second kernel). K tiles [keys][dh] and V^T tiles
// [dh][keys] are staged through LDS (double-buffered, rows padded by 16 bytes against bank
// conflicts) and shared by the 8 waves.
//
// The wave computes S^T = K Q^T, so a lane's 16 accumulator registers of a 32x32
// block all belong to ONE query row (column l%32) and 16 different keys
// (4*(l/32) + 8*j + i): the softmax row reductions are in-lane plus one exchange
// with lane l^32, and the probabilities are already laid out as the B operand of
// O^T = V^T P^T. The keys a lane holds for one 16-key MFMA step are
// {4c..4c+3, 8+4c..8+4c+3}; V^T is stored with that permutation (see
// chorus_v_transpose) so the matching A operand is a single 16-byte LDS read.
//
// The running maximum is only refreshed when a tile exceeds it by more than 8
// (in log2 units), which keeps exp2 arguments <= 8 and makes the accumulator
// rescale rare; the final division by the row sum makes the result exact either way.
#include "chorus_ops.h"
#include "common.h"

namespace chorus {
namespace {

constexpr int KT = 64;  // granularity of the key padding (the smaller of the two tile sizes)

// ---------------------------------------------------------------------------
// Ping-pong phases: 8 waves, one block of 32 query rows each, two groups of four
// waves (one wave of each group per SIMD). A wave alternates between a VALU phase
// (softmax of tile j) and an MFMA phase (O += V(j) P(j), then S(j+1) = K(j+1) Q^T),
// separated by workgroup barriers; group 1 runs one phase behind group 0, so on
// every SIMD one wave feeds the matrix pipe while the other runs the softmax.
//
// LDS holds two K and two V^T tiles. In its MFMA phase of tile j a wave first
// stores the registers it prefetched one iteration earlier (K(j+2) into the
// buffer S(j) was read from, V(j+1) into the buffer of V(j-1)), then issues the
// global loads for K(j+3) and V(j+2). Both groups have finished reading a buffer
// at least one barrier before either group overwrites it.
// ---------------------------------------------------------------------------
template <int DH, int KTL, bool COLSCALE>
__global__ __launch_bounds__(512, 2) void attention_pp_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ Vt,
    uint16_t* __restrict__ O, const float* __restrict__ col_scale, long Lq, long Lk, long LqPad, long LkPad, int H,
    int n_qtiles, float scale_log2) {
  constexpr int NT = 512;
  constexpr int KS = DH + 8, VS = KTL + 8;  // padded LDS row strides (elements)
  constexpr int KB = KTL / 32;                // 32-key blocks of S^T per tile
  constexpr int NKS = KTL / 16;               // 16-key MFMA steps of P V per tile
  constexpr int K_LD = KTL * (DH / 8) / NT;
  constexpr int V_LD = DH * (KTL / 8) / NT;
  constexpr int SK = DH / 16;
  constexpr int TD = DH / 32;
  constexpr int QROWS = 8 * 32;

  extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
  uint16_t* smk = reinterpret_cast<uint16_t*>(smem_raw);   // [2][KTL][KS]
  uint16_t* smv = smk + 2 * KTL * KS;                      // [2][DH][VS]

  const int tile_id = xcd_remap(blockIdx.x, H * n_qtiles);
  const int head = tile_id / n_qtiles;
  const int qt = tile_id - head * n_qtiles;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int group = wave >> 2;
  const int lrow = lane & 31, c = lane >> 5, lk = c * 8;
  const long q_wave0 = (long)qt * QROWS + wave * 32;

  const uint16_t* Kh = K + (long)head * LkPad * DH;
  const uint16_t* Vh = Vt + (long)head * DH * LkPad;

  bf16x8 qf[SK];
  {
    long q = q_wave0 + lrow;
    if (q > Lq - 1) q = Lq - 1;
    const uint16_t* qp = Q + ((long)head * LqPad + q) * DH + lk;
#pragma unroll
    for (int s = 0; s < SK; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qp + 16 * s);
  }

  f32x16 o[TD];
#pragma unroll
  for (int t = 0; t < TD; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[t][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const int ntiles = (int)((Lk + KTL - 1) / KTL);
  u32x4 rk[K_LD], rv[V_LD];

  auto load_k = [&](int kt) {
#pragma unroll
    for (int i = 0; i < K_LD; ++i)
      rk[i] = *reinterpret_cast<const u32x4*>(Kh + (long)kt * KTL * DH + (tid + NT * i) * 8);
  };
  auto load_v = [&](int kt) {
#pragma unroll
    for (int i = 0; i < V_LD; ++i) {
      int id = tid + NT * i, row = id / (KTL / 8), ch = id % (KTL / 8);
      rv[i] = *reinterpret_cast<const u32x4*>(Vh + (long)row * LkPad + (long)kt * KTL + ch * 8);
    }
  };
  auto store_k = [&](int buf) {
#pragma unroll
    for (int i = 0; i < K_LD; ++i) {
      int id = tid + NT * i, row = id / (DH / 8), ch = id % (DH / 8);
      *reinterpret_cast<u32x4*>(&smk[(buf * KTL + row) * KS + ch * 8]) = rk[i];
    }
  };
  auto store_v = [&](int buf) {
#pragma unroll
    for (int i = 0; i < V_LD; ++i) {
      int id = tid + NT * i, row = id / (KTL / 8), ch = id % (KTL / 8);
      *reinterpret_cast<u32x4*>(&smv[(buf * DH + row) * VS + ch * 8]) = rv[i];
    }
  };
  f32x16 s[KB];
  auto compute_s = [&](int buf) {
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < SK; ++ks) {
      bf16x8 kf[KB];
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
        kf[kb] = *reinterpret_cast<const bf16x8*>(&smk[(buf * KTL + 32 * kb + lrow) * KS + 16 * ks + lk]);
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb], qf[ks], s[kb], 0, 0, 0);
    }
  };

  // prologue: K(0), V(0), K(1) into LDS; K(2), V(1) into the prefetch registers
  load_k(0);
  load_v(0);
  store_k(0);
  store_v(0);
  if (ntiles > 1) {
    load_k(1);
    store_k(1);
    load_v(1);
  }
  if (ntiles > 2) load_k(2);
#pragma unroll
  for (int sI = 0; sI < SK; ++sI) asm volatile("" : "+v"(qf[sI]));  // Q fragments resident before the loop
  __syncthreads();
  compute_s(0);
  __syncthreads();
  if (group == 1) lds_barrier();  // run one phase behind group 0

  for (int j = 0; j < ntiles; ++j) {
    // ================= VALU phase: softmax of tile j =================
    __builtin_amdgcn_sched_barrier(0);
    const long key0 = (long)j * KTL + 4 * c;
    if (COLSCALE) {
      // a lane's keys come in runs of four: one 16-byte load per run (the runs that cross the end one key at a time)
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const long key = key0 + 32 * kb + 8 * q4;
          f32x4 cf;
          if (key + 3 < Lk) {
            cf = *reinterpret_cast<const f32x4*>(col_scale + key);
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) cf[i] = key + i < Lk ? col_scale[key + i] : 1.0f;
          }
#pragma unroll
          for (int i = 0; i < 4; ++i) s[kb][4 * q4 + i] *= cf[i] * scale_log2;
        }
    }
    if (j == ntiles - 1 && (Lk % KTL) != 0) {
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          long key = key0 + 32 * kb + 8 * (r >> 2) + (r & 3);
          if (key >= Lk) s[kb][r] = -INFINITY;
        }
    }
    float mx = s[0][0];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
    mx = fmaxf(mx, swap_halves(mx));
    const float mxs = COLSCALE ? mx : mx * scale_log2;
    if (__any(mxs > m_run + 8.0f)) {
      const float m_new = fmaxf(m_run, mxs);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int t = 0; t < TD; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][r] *= alpha;
    }
    bf16x8 pf[NKS];
    {
      const float mref = m_run;
      float lsum = 0.f;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float a = COLSCALE ? (s[kb][r] - mref) : __builtin_fmaf(s[kb][r], scale_log2, -mref);
          p[r] = __builtin_amdgcn_exp2f(a);
          lsum += p[r];
        }
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
          for (int e = 0; e < 8; ++e) pf[2 * kb + h2][e] = (bf16_t)p[8 * h2 + e];
      }
      l_run += lsum;
    }
    // the probabilities must exist before the barrier (otherwise the compiler sinks the
    // exponentials into the MFMA phase, which defeats the phase split)
#pragma unroll
    for (int i = 0; i < NKS; ++i) asm volatile("" : "+v"(pf[i]));
    __builtin_amdgcn_sched_barrier(0);
    lds_barrier();
    __builtin_amdgcn_sched_barrier(0);

    // ================= MFMA phase: O += V(j) P(j); S(j+1) = K(j+1) Q^T =================
    // Branch-free on purpose (one basic block the scheduler can pipeline): past the last
    // tiles the prefetch re-reads the final tile and the extra stores / S tile are never used.
    __builtin_amdgcn_s_setprio(1);
    store_k(j & 1);
    store_v((j + 1) & 1);
    load_k(j + 3 < ntiles ? j + 3 : ntiles - 1);
    load_v(j + 2 < ntiles ? j + 2 : ntiles - 1);
    {
      const int vb = j & 1;
#pragma unroll
      for (int t = 0; t < TD; ++t) {
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
          const bf16x8 vf = *reinterpret_cast<const bf16x8*>(&smv[(vb * DH + 32 * t + lrow) * VS + 16 * ks + lk]);
          o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ks], o[t], 0, 0, 0);
        }
      }
    }
    compute_s((j + 1) & 1);
    // issue order: LDS stores, global prefetch, then LDS operand reads kept 6 ahead of the MFMAs
    __builtin_amdgcn_sched_group_barrier(0x200, K_LD + V_LD, 0);
    __builtin_amdgcn_sched_group_barrier(0x020, K_LD + V_LD, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
    for (int i = 0; i < NKS * TD + KB * SK - 6; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 6, 0);
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
    lds_barrier();  // this wave's LDS stores are done; the global prefetch stays in flight
    __builtin_amdgcn_sched_barrier(0);
  }
  if (group == 0) lds_barrier();  // every wave executes the same number of barriers

  const int D = H * DH;
  const float l = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l;
  const long q = q_wave0 + lrow;
  if (q < Lq) {
    uint16_t* op = O + q * (long)D + head * DH + 4 * c;
#pragma unroll
    for (int t = 0; t < TD; ++t)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        uint2 w;
        w.x = pack_bf16x2(o[t][4 * jj + 0] * inv, o[t][4 * jj + 1] * inv);
        w.y = pack_bf16x2(o[t][4 * jj + 2] * inv, o[t][4 * jj + 3] * inv);
        *reinterpret_cast<uint2*>(op + 32 * t + 8 * jj) = w;
      }
  }
}

// ---------------------------------------------------------------------------
// The same ping-pong kernel on v_mfma_f32_16x16x32_bf16, 128-key tiles, no column scale. Per flop this shape writes
// half the accumulator registers of the 32x32x16 one and a result block is accumulated by four MFMAs in a row (the
// whole head dimension or the whole key tile), which is what the power-managed part rewards.
//
// A wave still owns 32 query rows, as two blocks of 16 (rb). Lane l: query row l % 16 of each block, and of every
// 16 x 16 result block the four rows 4 g .. 4 g + 3, g = l / 16.
//   S^T block kb (16 keys x 16 query rows, kb = 0..7 of a 128-key tile): the K fragment's row r is key
//   32 (kb / 2) + 16 (r / 8) + 8 (kb % 2) + r % 8 of the tile, so the lane holds keys 32 (kb / 2) + 16 (g / 2) +
//   8 (kb % 2) + 4 (g % 2) + i. For a 32-key step of O^T += V^T P^T (blocks kb = 2 c, 2 c + 1) these eight keys are
//   {4 (g % 2) .. + 3, 8 + 4 (g % 2) .. + 3} of the 16-key group 2 c + g / 2: exactly the eight consecutive
//   positions 8 g .. 8 g + 7 of the step in the stored V^T order (see chorus_v_transpose), so the V operand is one
//   16-byte LDS read and the lane's probabilities are its B operand as they stand.
// LDS rows are padded by 32 bytes: with 16 rows x 4 chunks per fragment read that stride is free of bank conflicts.
// Two things leave the vector pipe, which in this kernel is as loaded as the matrix pipe: the softmax row sums are
// taken by the matrix pipe (one more result block per 16 query rows whose V operand is all ones, so the sum is over
// the same bf16-rounded probabilities that weight V and the weights of a row add up to exactly one), and the global
// prefetch of the next tiles is issued at the start of the softmax phase instead of the MFMA phase.
// ---------------------------------------------------------------------------
// KIND 0 and 1 are the same code: 1 gives launches with a key sequence other than the query sequence (the text
// cross-attention) a kernel name of their own, so that a kernel profile lists self- and cross-attention separately.
// KIND 2 multiplies the logit of key j by col_scale[j] (TGAA's key amplification, Eq. 2, applied to the logit): the
// S^T accumulators then start at zero and one multiply-add per logit applies the factor and, with PRE, the reference.
template <int DH, bool PRE, int RB, int KIND>
__global__ __launch_bounds__(512, 2) void attention_pp16_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ Vt,
    uint16_t* __restrict__ O, const float* __restrict__ col_scale, long Lq, long Lk, long LqPad, long LkPad, int H,
    int n_qtiles, int tile_base, float scale_log2) {
  constexpr bool CS = KIND == 2;
  constexpr int NT = 512;
  constexpr int KTL = 128;
  constexpr int KS = DH + 16, VS = KTL + 16;  // padded LDS row strides (elements)
  constexpr int KB = KTL / 16;                 // 16-key blocks of S^T per tile
  constexpr int NC = KTL / 32;                 // 32-key MFMA steps of P V per tile
  constexpr int KC = DH / 32;                  // 32-wide steps over the head dimension
  constexpr int DB = DH / 16;                  // 16-row blocks of O^T
  constexpr int K_LD = KTL * (DH / 8) / NT;
  constexpr int V_LD = DH * (KTL / 8) / NT;
  constexpr int QROWS = 8 * 16 * RB;  // RB blocks of 16 query rows per wave

  extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
  uint16_t* smk = reinterpret_cast<uint16_t*>(smem_raw);   // [2][KTL][KS]
  uint16_t* smv = smk + 2 * KTL * KS;                      // [2][DH][VS]

  // this launch covers the tiles tile_base .. tile_base + gridDim.x - 1 of the H * n_qtiles of its tile size
  const int tile_id = tile_base + xcd_remap(blockIdx.x, gridDim.x);
  const int head = tile_id / n_qtiles;
  const int qt = tile_id - head * n_qtiles;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int group = wave >> 2;
  const int lq = lane & 15, g = lane >> 4;
  const long q_wave0 = (long)qt * QROWS + wave * 16 * RB;

  const uint16_t* Kh = K + (long)head * LkPad * DH;
  const uint16_t* Vh = Vt + (long)head * DH * LkPad;

  bf16x8 qf[RB][KC];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    long q = q_wave0 + 16 * rb + lq;
    if (q > Lq - 1) q = Lq - 1;
    const uint16_t* qp = Q + ((long)head * LqPad + q) * DH + 8 * g;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) qf[rb][kc] = *reinterpret_cast<const bf16x8*>(qp + 32 * kc);
  }

  f32x4 o[DB][RB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) o[db][rb] = f32x4{0.f, 0.f, 0.f, 0.f};
  // PRE: Q arrives multiplied by log2(e) / sqrt(dh) and the S^T accumulators start at minus the running reference, so
  // a logit leaves the MFMA as the exponent of its probability; the reference starts at 0 and the first tile sets it.
  float m_run[RB];
  f32x4 lacc[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    m_run[rb] = PRE ? 0.f : -INFINITY;
    lacc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (bf16_t)1.0f;

  const int ntiles = (int)((Lk + KTL - 1) / KTL);
  u32x4 rk[K_LD], rv[V_LD];

  auto load_k = [&](int kt) {
#pragma unroll
    for (int i = 0; i < K_LD; ++i)
      rk[i] = *reinterpret_cast<const u32x4*>(Kh + (long)kt * KTL * DH + (tid + NT * i) * 8);
  };
  auto load_v = [&](int kt) {
#pragma unroll
    for (int i = 0; i < V_LD; ++i) {
      int id = tid + NT * i, row = id / (KTL / 8), ch = id % (KTL / 8);
      rv[i] = *reinterpret_cast<const u32x4*>(Vh + (long)row * LkPad + (long)kt * KTL + ch * 8);
    }
  };
  auto store_k = [&](int buf) {
#pragma unroll
    for (int i = 0; i < K_LD; ++i) {
      int id = tid + NT * i, row = id / (DH / 8), ch = id % (DH / 8);
      *reinterpret_cast<u32x4*>(&smk[(buf * KTL + row) * KS + ch * 8]) = rk[i];
    }
  };
  auto store_v = [&](int buf) {
#pragma unroll
    for (int i = 0; i < V_LD; ++i) {
      int id = tid + NT * i, row = id / (KTL / 8), ch = id % (KTL / 8);
      *reinterpret_cast<u32x4*>(&smv[(buf * DH + row) * VS + ch * 8]) = rv[i];
    }
  };
  // LDS row of the K tile that fragment row lane % 16 of block kb stands for
  const int krow0 = 16 * (lq >> 3) + (lq & 7);
  f32x4 s[KB][RB];
  auto compute_s = [&](int buf) {
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
      bf16x8 kf[KC];
      const int row = 32 * (kb >> 1) + 8 * (kb & 1) + krow0;
#pragma unroll
      for (int kc = 0; kc < KC; ++kc)
        kf[kc] = *reinterpret_cast<const bf16x8*>(&smk[(buf * KTL + row) * KS + 32 * kc + 8 * g]);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const float a0 = (PRE && !CS) ? -m_run[rb] : 0.f;
        f32x4 acc = {a0, a0, a0, a0};
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kc], qf[rb][kc], acc, 0, 0, 0);
        s[kb][rb] = acc;
      }
    }
  };

  // prologue: K(0), V(0), K(1) into LDS; K(2), V(1) into the prefetch registers
  load_k(0);
  load_v(0);
  store_k(0);
  store_v(0);
  if (ntiles > 1) {
    load_k(1);
    store_k(1);
  }
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) asm volatile("" : "+v"(qf[rb][kc]));  // Q fragments resident before the loop
  __syncthreads();
  compute_s(0);
  __syncthreads();
  if (group == 1) lds_barrier();  // run one phase behind group 0

  for (int j = 0; j < ntiles; ++j) {
    // ================= VALU phase: softmax of tile j =================
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (CS) {
      // the column factors of this tile are fetched and applied before the prefetch is issued: loads return in order,
      // and the 32 registers they take are free again when the prefetch needs its own
      const int key0 = j * KTL + 16 * (g >> 1) + 4 * (g & 1);
      const int lk = (int)Lk;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        const int key = key0 + 32 * (kb >> 1) + 8 * (kb & 1);
        f32x4 cf;
        if (key + 3 < lk) {
          cf = *reinterpret_cast<const f32x4*>(col_scale + key);
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) cf[i] = key + i < lk ? col_scale[key + i] : 1.0f;
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            s[kb][rb][i] = PRE ? __builtin_fmaf(s[kb][rb][i], cf[i], -m_run[rb]) : s[kb][rb][i] * cf[i];
        if (kb % 2 == 1) __builtin_amdgcn_sched_barrier(0);  // two factors in flight at a time: there are no registers for eight
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // the global prefetch of the tiles that the next MFMA phase stores: K(j+2), V(j+1) (past the end the last tile again)
    load_k(j + 2 < ntiles ? j + 2 : ntiles - 1);
    load_v(j + 1 < ntiles ? j + 1 : ntiles - 1);
    if (j == ntiles - 1 && (Lk % KTL) != 0) {
      const long key0 = (long)j * KTL + 16 * (g >> 1) + 4 * (g & 1);
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const long key = key0 + 32 * (kb >> 1) + 8 * (kb & 1) + i;
          if (key >= Lk) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) s[kb][rb][i] = -INFINITY;
          }
        }
    }
    float mxs[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      float mx = s[0][rb][0];
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int i = 0; i < 4; ++i) mx = fmaxf(mx, s[kb][rb][i]);
      mx = fmaxf(mx, swap_rows16(mx));
      mx = fmaxf(mx, swap_halves(mx));
      mxs[rb] = PRE ? mx : mx * scale_log2;
    }
    if constexpr (PRE) {
      // logits are relative to the reference already: move it when a row exceeds it by more than 8, and on the first tile
      bool move = false;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) move = move || mxs[rb] > 8.0f;
      if (__any(move) || j == 0) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          const float delta = j == 0 ? mxs[rb] : fmaxf(mxs[rb], 0.f);
          const float alpha = j == 0 ? 1.0f : __builtin_amdgcn_exp2f(-delta);  // nothing is accumulated before the first tile
          m_run[rb] += delta;
          lacc[rb] *= alpha;
#pragma unroll
          for (int db = 0; db < DB; ++db) o[db][rb] *= alpha;
#pragma unroll
          for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int i = 0; i < 4; ++i) s[kb][rb][i] -= delta;
        }
      }
    } else {
      bool move = false;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) move = move || mxs[rb] > m_run[rb] + 8.0f;
      if (__any(move)) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const float m_new = fmaxf(m_run[rb], mxs[rb]);
        const float alpha = __builtin_amdgcn_exp2f(m_run[rb] - m_new);
        m_run[rb] = m_new;
        lacc[rb] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db) o[db][rb] *= alpha;
      }
      }
    }
    bf16x8 pf[NC][RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const float mref = m_run[rb];
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float p = PRE ? __builtin_amdgcn_exp2f(s[2 * c + b][rb][i])
                                : __builtin_amdgcn_exp2f(__builtin_fmaf(s[2 * c + b][rb][i], scale_log2, -mref));
            pf[c][rb][4 * b + i] = (bf16_t)p;
          }
    }
    // the probabilities must exist before the barrier (otherwise the compiler sinks the
    // exponentials into the MFMA phase, which defeats the phase split)
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) asm volatile("" : "+v"(pf[c][rb]));
    __builtin_amdgcn_sched_barrier(0);
    lds_barrier();
    __builtin_amdgcn_sched_barrier(0);

    // ================= MFMA phase: O += V(j) P(j); S(j+1) = K(j+1) Q^T =================
    __builtin_amdgcn_s_setprio(1);
    store_k(j & 1);
    store_v((j + 1) & 1);
    {
      const int vb = j & 1;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        bf16x8 vf[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c)
          vf[c] = *reinterpret_cast<const bf16x8*>(&smv[(vb * DH + 16 * db + lq) * VS + 32 * c + 8 * g]);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int c = 0; c < NC; ++c) o[db][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[c], pf[c][rb], o[db][rb], 0, 0, 0);
      }
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int c = 0; c < NC; ++c) lacc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pf[c][rb], lacc[rb], 0, 0, 0);
    }
    compute_s((j + 1) & 1);
    // issue order: LDS stores, then LDS operand reads kept ahead of the MFMAs (one read feeds two)
    constexpr int kAhead = 6;  // more reads in flight cost the registers the schedule needs; fewer expose LDS latency
    __builtin_amdgcn_sched_group_barrier(0x200, K_LD + V_LD, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, kAhead, 0);
#pragma unroll
    for (int i = 0; i < DB * NC + KB * KC - kAhead; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, RB, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, RB * kAhead + RB * NC, 0);
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
    lds_barrier();  // this wave's LDS stores are done
    __builtin_amdgcn_sched_barrier(0);
  }
  if (group == 0) lds_barrier();  // every wave executes the same number of barriers

  const int D = H * DH;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const float l = lacc[rb][0];
    const float inv = 1.0f / l;
    const long q = q_wave0 + 16 * rb + lq;
    if (q < Lq) {
      uint16_t* op = O + q * (long)D + head * DH + 4 * g;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        uint2 w;
        w.x = pack_bf16x2(o[db][rb][0] * inv, o[db][rb][1] * inv);
        w.y = pack_bf16x2(o[db][rb][2] * inv, o[db][rb][3] * inv);
        *reinterpret_cast<uint2*>(op + 16 * db) = w;
      }
    }
  }
}

// One launch of the 16x16x32 kernel with RB blocks of 16 query rows per wave over the tiles tile_base .. + ntile - 1.
template <int DH, bool PRE, int RB, int KIND>
int32_t launch_attn_pp16_tiles(const uint16_t* Q, const uint16_t* K, const uint16_t* Vt, uint16_t* O, const float* cs,
                               long Lq, long Lk, long LqPad, long LkPad, int H, long nqt, long tile_base, long ntile,
                               hipStream_t s) {
  size_t smem = 2 * ((size_t)128 * (DH + 16) + (size_t)DH * (128 + 16)) * sizeof(uint16_t);
  auto kern = attention_pp16_kernel<DH, PRE, RB, KIND>;
  static DynLdsOnce once;  // the raised dynamic-LDS limit is a per-device property of the kernel
  CHK_STATUS(once.ensure(reinterpret_cast<const void*>(kern), (int)smem));
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);
  hipLaunchKernelGGL(kern, dim3((unsigned)ntile), dim3(512), smem, s, Q, K, Vt, O, cs, Lq, Lk, LqPad, LkPad, H,
                     (int)nqt, (int)tile_base, scale_log2);
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

// 256 query rows per workgroup. One workgroup fits a CU, so a launch runs in rounds of as many workgroups as the device
// has CUs. When the last round would be at most half full, its tiles run as workgroups of 128 rows instead (one block
// of 16 rows per wave: the same K / V stream for half the arithmetic, 0.63-0.67 of a full workgroup's time), twice as
// many of them, in a second launch behind the first: the partly filled round then takes two thirds of a full one.
template <int DH, bool PRE, int KIND>
int32_t launch_attn_pp16_kind(const uint16_t* Q, const uint16_t* K, const uint16_t* Vt, uint16_t* O, const float* cs, long Lq,
                              long Lk, long LqPad, long LkPad, int H, hipStream_t s) {
  const long nqt = (Lq + 255) / 256;
  const long tiles = nqt * H;
  if (2 * tiles > 0x7fffffffL) return CHORUS_E_SHAPE;
  int dev = 0, cus = 0;
  CHORUS_HIP(hipGetDevice(&dev));
  CHORUS_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  const long tail = cus > 0 ? tiles % cus : 0;
  if (tiles > cus && tail > 0 && 2 * tail <= cus) {
    CHK_STATUS((launch_attn_pp16_tiles<DH, PRE, 2, KIND>(Q, K, Vt, O, cs, Lq, Lk, LqPad, LkPad, H, nqt, 0, tiles - tail, s)));
    return launch_attn_pp16_tiles<DH, PRE, 1, KIND>(Q, K, Vt, O, cs, Lq, Lk, LqPad, LkPad, H, 2 * nqt, 2 * (tiles - tail),
                                                    2 * tail, s);
  }
  return launch_attn_pp16_tiles<DH, PRE, 2, KIND>(Q, K, Vt, O, cs, Lq, Lk, LqPad, LkPad, H, nqt, 0, tiles, s);
}

template <int DH, bool PRE>
int32_t launch_attn_pp16(const uint16_t* Q, const uint16_t* K, const uint16_t* Vt, uint16_t* O, const float* cs, long Lq,
                         long Lk, long LqPad, long LkPad, int H, hipStream_t s) {
  if (cs) return launch_attn_pp16_kind<DH, PRE, 2>(Q, K, Vt, O, cs, Lq, Lk, LqPad, LkPad, H, s);
  return Lq == Lk ? launch_attn_pp16_kind<DH, PRE, 0>(Q, K, Vt, O, cs, Lq, Lk, LqPad, LkPad, H, s)
                  : launch_attn_pp16_kind<DH, PRE, 1>(Q, K, Vt, O, cs, Lq, Lk, LqPad, LkPad, H, s);
}

template <int DH, int KTL, bool CS>
int32_t launch_attn_pp(const uint16_t* Q, const uint16_t* K, const uint16_t* Vt, uint16_t* O, const float* cs, long Lq,
                       long Lk, long LqPad, long LkPad, int H, hipStream_t s) {
  long nqt = (Lq + 255) / 256;
  if (nqt * H > 0x7fffffffL) return CHORUS_E_SHAPE;
  size_t smem = 2 * ((size_t)KTL * (DH + 8) + (size_t)DH * (KTL + 8)) * sizeof(uint16_t);
  auto kern = attention_pp_kernel<DH, KTL, CS>;
  static DynLdsOnce once;  // the raised dynamic-LDS limit is a per-device property of the kernel
  CHK_STATUS(once.ensure(reinterpret_cast<const void*>(kern), (int)smem));
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)DH);
  hipLaunchKernelGGL(kern, dim3((unsigned)(nqt * H)), dim3(512), smem, s, Q, K, Vt, O, cs, Lq, Lk, LqPad, LkPad, H,
                     (int)nqt, scale_log2);
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

}  // namespace
}  // namespace chorus

using namespace chorus;

// variant: 0 = default choice; 3 = 64-key tiles on 32x32x16 MFMAs; 5 = 128-key tiles on 16x16x32 MFMAs
// (LkPad % 128 == 0); 6 = the same on pre-scaled queries
extern "C" int32_t chorus_attention(const uint16_t* Q, const uint16_t* K, const uint16_t* Vt, uint16_t* O,
                                    const float* col_scale, int64_t Lq, int64_t Lk, int64_t LqPad, int64_t LkPad,
                                    int32_t H, int32_t dh, int32_t variant, void* stream) {
  if (Lq < 0 || Lk < 0 || H <= 0) return CHORUS_E_ARG;
  if (variant != 0 && variant != 3 && variant != 5 && variant != 6) return CHORUS_E_ARG;
  if (Lq == 0) return CHORUS_OK;
  if (Lk < 1) return CHORUS_E_SHAPE;
  if (!Q || !K || !Vt || !O) return CHORUS_E_ARG;
  if ((dh != 64 && dh != 128) || LkPad % KT || LkPad < Lk || LqPad < Lq || LkPad > 0x7fffffffL) return CHORUS_E_SHAPE;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(Vt) || !aligned16(O) || !aligned16(col_scale)) return CHORUS_E_ARG;
  hipStream_t s = (hipStream_t)stream;
  const bool cs = col_scale != nullptr;
  // 128-key tiles on the 16x16x32 kernel when the keys are long enough and the padding allows
  if (variant == 0) variant = CHORUS_ATTENTION_LONG_KEYS(Lk, LkPad) ? 5 : 3;
  if (variant == 5 || variant == 6) {
    if (LkPad % 128) return CHORUS_E_SHAPE;
    if (variant == 6)
      return dh == 128 ? launch_attn_pp16<128, true>(Q, K, Vt, O, col_scale, Lq, Lk, LqPad, LkPad, H, s)
                       : launch_attn_pp16<64, true>(Q, K, Vt, O, col_scale, Lq, Lk, LqPad, LkPad, H, s);
    return dh == 128 ? launch_attn_pp16<128, false>(Q, K, Vt, O, col_scale, Lq, Lk, LqPad, LkPad, H, s)
                     : launch_attn_pp16<64, false>(Q, K, Vt, O, col_scale, Lq, Lk, LqPad, LkPad, H, s);
  }
  if (dh == 128)
    return cs ? launch_attn_pp<128, 64, true>(Q, K, Vt, O, col_scale, Lq, Lk, LqPad, LkPad, H, s)
              : launch_attn_pp<128, 64, false>(Q, K, Vt, O, col_scale, Lq, Lk, LqPad, LkPad, H, s);
  return cs ? launch_attn_pp<64, 64, true>(Q, K, Vt, O, col_scale, Lq, Lk, LqPad, LkPad, H, s)
            : launch_attn_pp<64, 64, false>(Q, K, Vt, O, col_scale, Lq, Lk, LqPad, LkPad, H, s);
}
