// Batched top-k retrieval (Sec. 3.1 "Full Reuse" for a queue of requests): the k best cache
// entries by cosine similarity for each of Q prompt embeddings, with ONE pass over the
// [N, d] fp32 cache per 32 queries instead of one per query. The scan is a [N, d] x [d, Q]
// contraction in fp32, so it runs on the fp32 matrix pipe (16x16x4), which at 16-32 queries
// needs about the cycles that HBM needs to deliver the cache rows; row norms are accumulated
// from the same registers.
#include "common.h"

namespace chorus {
namespace {

constexpr int kRB = 1;        // 16-row blocks per wave
constexpr int kBR = 64 * kRB;  // cache rows per workgroup, 16 kRB per wave
constexpr int kBK = 64;       // floats of every row per step (256 bytes: two full cache lines)
constexpr int kLS = kBK + 4;  // LDS row stride in floats (16-byte aligned, staggers the banks)

struct BatchPlan {
  int tiles;             // row tiles
  int KS;                // slices along d
  int chunks_per_slice;  // kBK-float steps per slice
};

inline BatchPlan plan_batch(long N, int d) {
  BatchPlan p;
  p.tiles = (int)((N + kBR - 1) / kBR);
  const int nchunks = (d + kBK - 1) / kBK;
  // enough workgroups to put four on each of 256 CUs; partial sums of the slices are added in a fixed order afterwards
  int want = p.tiles > 0 ? (1024 + p.tiles - 1) / p.tiles : 1;
  if (want < 1) want = 1;
  if (want > nchunks) want = nchunks;
  if (want > 16) want = 16;  // every slice writes and re-reads its own partial sums
  p.chunks_per_slice = (nchunks + want - 1) / want;
  p.KS = (nchunks + p.chunks_per_slice - 1) / p.chunks_per_slice;
  return p;
}

// part_dot [KS][Qp][Npad] (row fastest, Npad = N rounded up to 128), part_cc [KS][Npad]; Qp = 16 * QB
template <int QB>
__global__ __launch_bounds__(256) void lookup_batch_scores_kernel(const float* __restrict__ cache,
                                                                  const float* __restrict__ queries,
                                                                  float* __restrict__ part_dot,
                                                                  float* __restrict__ part_cc, long N, int d, int Q,
                                                                  int chunks_per_slice) {
  constexpr int QP = 16 * QB;
  __shared__ __attribute__((aligned(16))) float sA[kBR * kLS];
  __shared__ __attribute__((aligned(16))) float sB[QP * kLS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const long row0 = (long)blockIdx.x * kBR;
  const long Npad = (long)gridDim.x * kBR;
  const int ks = blockIdx.y;
  const int c0 = ks * chunks_per_slice;
  const int nchunks = (d + kBK - 1) / kBK;
  const int c1 = c0 + chunks_per_slice < nchunks ? c0 + chunks_per_slice : nchunks;

  // loader role: 16 threads per row segment of 256 bytes
  const int lcol = tid & 15, lrow = tid >> 4;
  f32x4 ra[2][4 * kRB], rb[2][QB];  // two chunks in flight
  auto load_chunk = [&](int st, int c) {
    const int k = c * kBK + 4 * lcol;
#pragma unroll
    for (int i = 0; i < 4 * kRB; ++i) {
      const long r = row0 + lrow + 16 * i;
      const bool ok = r < N && k < d;
      const float* p = cache + (ok ? r : 0) * (long)d + (ok ? k : 0);
      f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
      ra[st][i] = ok ? v : f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int i = 0; i < QB; ++i) {
      const int q = lrow + 16 * i;
      const bool ok = q < Q && k < d;
      const float* p = queries + (long)(ok ? q : 0) * d + (ok ? k : 0);
      f32x4 v = *reinterpret_cast<const f32x4*>(p);
      rb[st][i] = ok ? v : f32x4{0.f, 0.f, 0.f, 0.f};
    }
  };
  auto store_chunk = [&](int st) {
#pragma unroll
    for (int i = 0; i < 4 * kRB; ++i) *reinterpret_cast<f32x4*>(&sA[(lrow + 16 * i) * kLS + 4 * lcol]) = ra[st][i];
#pragma unroll
    for (int i = 0; i < QB; ++i) *reinterpret_cast<f32x4*>(&sB[(lrow + 16 * i) * kLS + 4 * lcol]) = rb[st][i];
  };

  // compute role: a wave owns 32 rows = two 16-row blocks; lane = (row or query l % 16, k quarter l / 16)
  const int l16 = lane & 15, kq = lane >> 4;
  f32x4 acc[kRB][QB];
#pragma unroll
  for (int r = 0; r < kRB; ++r)
#pragma unroll
    for (int q = 0; q < QB; ++q) acc[r][q] = f32x4{0.f, 0.f, 0.f, 0.f};
  float cc[kRB] = {};

  // chunk c + 1 is already in flight when chunk c is stored, and chunk c + 2 is requested right after: two chunks
  // (64 KB per workgroup) are on their way during the MFMAs. Past the slice the loads are masked to zeros.
  auto step = [&](int st, int c) {
    __syncthreads();  // the previous step's reads are done
    store_chunk(st);
    __syncthreads();
    if (c + 2 < c1) load_chunk(st, c + 2);
#pragma unroll
    for (int j = 0; j < kBK / 16; ++j) {
      f32x4 a[kRB], b[QB];
#pragma unroll
      for (int r = 0; r < kRB; ++r) a[r] = *reinterpret_cast<const f32x4*>(&sA[(16 * kRB * wave + 16 * r + l16) * kLS + 16 * j + 4 * kq]);
#pragma unroll
      for (int q = 0; q < QB; ++q) b[q] = *reinterpret_cast<const f32x4*>(&sB[(16 * q + l16) * kLS + 16 * j + 4 * kq]);
#pragma unroll
      for (int r = 0; r < kRB; ++r) {
        cc[r] += a[r][0] * a[r][0] + a[r][1] * a[r][1] + a[r][2] * a[r][2] + a[r][3] * a[r][3];
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int q = 0; q < QB; ++q) acc[r][q] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r][e], b[q][e], acc[r][q], 0, 0, 0);
      }
    }
  };
  if (c0 < c1) load_chunk(0, c0);
  if (c0 + 1 < c1) load_chunk(1, c0 + 1);
  for (int c = c0; c < c1; c += 2) {
    step(0, c);
    if (c + 1 < c1) step(1, c + 1);
  }
  // row norms: the four k quarters of a row sit in lanes l16, l16 + 16, l16 + 32, l16 + 48
#pragma unroll
  for (int r = 0; r < kRB; ++r) {
    cc[r] += __shfl_xor(cc[r], 16, 64);
    cc[r] += __shfl_xor(cc[r], 32, 64);
    const long row = row0 + 16 * kRB * wave + 16 * r + l16;
    if (kq == 0) part_cc[(long)ks * Npad + row] = cc[r];
  }
  // accumulator elements 0..3 of lane (l16, kq): rows 4 kq .. 4 kq + 3 of the block, query l16 (rows past N hold zeros)
#pragma unroll
  for (int r = 0; r < kRB; ++r)
#pragma unroll
    for (int q = 0; q < QB; ++q) {
      const long row = row0 + 16 * kRB * wave + 16 * r + 4 * kq;
      *reinterpret_cast<f32x4*>(&part_dot[((long)ks * QP + 16 * q + l16) * Npad + row]) = acc[r][q];
    }
}

// dot[u], cc[u] (u < RU) += the partial sums of entry j + STRIDE u over the KS slices, in ascending slice order
// whatever the grouping: G slices x RU entries x 2 loads are in flight at a time.
template <int RU, int G, int RMAX, int STRIDE>
__device__ __forceinline__ void sum_slices(const float* __restrict__ part_dot, const float* __restrict__ part_cc, int KS,
                                           int QP, int q, long Npad, long j, long N, float (&dot)[RMAX], float (&cc)[RMAX]) {
  for (int ks0 = 0; ks0 < KS; ks0 += G) {
    float pd[G][RU], pc[G][RU];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const int ks = ks0 + g < KS ? ks0 + g : KS - 1;
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const long ju = j + (long)STRIDE * u;
        const long jj = ju < N ? ju : N - 1;
        pd[g][u] = part_dot[((long)ks * QP + q) * Npad + jj];
        pc[g][u] = part_cc[(long)ks * Npad + jj];
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int u = 0; u < RU; ++u) {
        const bool live = ks0 + g < KS;
        dot[u] += live ? pd[g][u] : 0.f;
        cc[u] += live ? pc[g][u] : 0.f;
      }
  }
}

constexpr int kWaveK = 64;  // up to this k the selection runs without a barrier per position

// Final scores of all queries: score[q][j] = (partial dots summed in slice order) / (|c_j| |q|), -inf for zero norms
// and NaN. Grid (row blocks of 1024, queries): spread over the chip, because one workgroup per query would pull its
// KS slices (half a megabyte at 4096 entries) through a single compute unit.
__global__ __launch_bounds__(256) void lookup_batch_final_kernel(const float* __restrict__ part_dot,
                                                                 const float* __restrict__ part_cc,
                                                                 const float* __restrict__ queries,
                                                                 float* __restrict__ scores, long N, long Npad, int d,
                                                                 int QP, int KS) {
  constexpr int R = 4;
  __shared__ float sq[4];
  const int q = blockIdx.y;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  float qq = 0.f;
  for (int i = tid; i < d; i += 256) {
    const float v = queries[(long)q * d + i];
    qq += v * v;
  }
  qq = wave_sum(qq);
  if (lane == 0) sq[wave] = qq;
  __syncthreads();
  const float qn = sqrtf(sq[0] + sq[1] + sq[2] + sq[3]);
  const long j0 = (long)blockIdx.x * (256 * R) + tid;
  float dot[R], cc[R];
#pragma unroll
  for (int u = 0; u < R; ++u) dot[u] = cc[u] = 0.f;
  sum_slices<R, 8, R, 256>(part_dot, part_cc, KS, QP, q, Npad, j0, N, dot, cc);
#pragma unroll
  for (int u = 0; u < R; ++u) {
    const long j = j0 + 256L * u;
    const float den = sqrtf(cc[u]) * qn;
    float v = den > 0.f ? dot[u] / den : -INFINITY;
    if (!(v == v)) v = -INFINITY;
    if (j < N) scores[(long)q * Npad + j] = v;
  }
}

// One workgroup per query: k rounds over its final scores, each picking the best entry that comes after the
// previous winner in the order (score descending, index ascending). REG: the scores of a thread live in registers
// (N <= 8 * 1024), else they are re-read from `scores`.
template <bool REG>
__global__ __launch_bounds__(1024) void lookup_topk_kernel(const float* __restrict__ scores, long N, long Npad, int k,
                                                           float tau, int32_t* __restrict__ out_idx,
                                                           float* __restrict__ out_score, int32_t* __restrict__ out_hit) {
  constexpr int R = 8;
  __shared__ float sv[2][16];
  __shared__ int si[2][16];  // N < 2^31 entries per call
  __shared__ float cv[16][kWaveK];  // small k: the kWaveK best of every wave, best first
  __shared__ int ci[16][kWaveK];
  const int q = blockIdx.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float* sc = scores + (long)q * Npad;
  float mine[R];
#pragma unroll
  for (int u = 0; u < R; ++u) {
    const long j = tid + 1024L * u;
    mine[u] = (REG && j < N) ? sc[j] : -INFINITY;
  }
  unsigned taken = 0;  // REG: bit u set = this thread's entry u has been output
  if (k <= kWaveK) {
    // Small k without a workgroup barrier per position: every wave first lists the k best of ITS entries (rounds of
    // in-wave exchanges only), then the first wave merges the 16 sorted lists. The k best overall are among them.
    float ps_w = INFINITY;
    int pj_w = -1;
    for (int r = 0; r < k; ++r) {
      float best = -INFINITY;
      int bi = -1;
      if (REG) {
#pragma unroll
        for (int u = 0; u < R; ++u) {
          const int j = tid + 1024 * u;
          if (j < N && !(taken & (1u << u)) && (bi < 0 || mine[u] > best)) {
            best = mine[u];
            bi = j;
          }
        }
      } else {
        for (long j = tid; j < N; j += 1024) {
          const float v = sc[j];
          const bool eligible = r == 0 || v < ps_w || (v == ps_w && j > pj_w);
          if (eligible && (bi < 0 || v > best)) {
            best = v;
            bi = (int)j;
          }
        }
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const float ob = __shfl_xor(best, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (oi >= 0 && (bi < 0 || ob > best || (ob == best && oi < bi))) {
          best = ob;
          bi = oi;
        }
      }
      if (lane == 0) {
        cv[wave][r] = best;
        ci[wave][r] = bi;
      }
      ps_w = best;
      pj_w = bi;
      if (REG && bi >= 0 && (bi & 1023) == tid) taken |= 1u << (unsigned)(bi >> 10);
      if (bi < 0) {  // this wave's entries are used up: the rest of its list is empty
        for (int rr = r + 1 + lane; rr < k; rr += 64) ci[wave][rr] = -1;
        break;
      }
    }
    __syncthreads();
    if (wave == 0) {
      int head = 0;  // lanes 0..15: position in the list of wave `lane`
      for (int r = 0; r < k; ++r) {
        int i = (lane < 16 && head < k) ? ci[lane][head] : -1;
        float b = i >= 0 ? cv[lane][head] : -INFINITY;
        const int mine_i = i;
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) {
          const float ob = __shfl_xor(b, o, 64);
          const int oi = __shfl_xor(i, o, 64);
          if (oi >= 0 && (i < 0 || ob > b || (ob == b && oi < i))) {
            b = ob;
            i = oi;
          }
        }
        b = __shfl(b, 0, 64);
        i = __shfl(i, 0, 64);
        if (lane == 0) {
          out_idx[(long)q * k + r] = i;
          out_score[(long)q * k + r] = i >= 0 ? b : -INFINITY;
          if (r == 0) out_hit[q] = (i >= 0 && b >= tau) ? 1 : 0;
        }
        if (i >= 0 && mine_i == i) ++head;  // the winner's list moves on
      }
    }
    return;
  }
  float ps = INFINITY;
  int pj = -1;
  for (int r = 0; r < k; ++r) {
    float best = -INFINITY;
    int bi = -1;
    if (REG) {
#pragma unroll
      for (int u = 0; u < R; ++u) {
        const int j = tid + 1024 * u;
        if (j < N && !(taken & (1u << u)) && (bi < 0 || mine[u] > best)) {
          best = mine[u];
          bi = j;
        }
      }
    } else {
      for (long j = tid; j < N; j += 1024) {
        const float v = sc[j];
        const bool eligible = r == 0 || v < ps || (v == ps && j > pj);
        if (eligible && (bi < 0 || v > best)) {  // ascending j: the first of equal values stays
          best = v;
          bi = (int)j;
        }
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ob = __shfl_xor(best, o, 64);
      const int oi = __shfl_xor(bi, o, 64);
      if (oi >= 0 && (bi < 0 || ob > best || (ob == best && oi < bi))) {
        best = ob;
        bi = oi;
      }
    }
    const int buf = r & 1;  // alternating buffers: one barrier per round
    if (lane == 0) {
      sv[buf][wave] = best;
      si[buf][wave] = bi;
    }
    __syncthreads();
    // every wave reduces the 16 candidates again: lane w holds candidate w
    float b = lane < 16 ? sv[buf][lane] : -INFINITY;
    int i = lane < 16 ? si[buf][lane] : -1;
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) {
      const float ob = __shfl_xor(b, o, 64);
      const int oi = __shfl_xor(i, o, 64);
      if (oi >= 0 && (i < 0 || ob > b || (ob == b && oi < i))) {
        b = ob;
        i = oi;
      }
    }
    b = __shfl(b, 0, 64);
    i = __shfl(i, 0, 64);
    if (tid == 0) {
      out_idx[(long)q * k + r] = i;
      out_score[(long)q * k + r] = i >= 0 ? b : -INFINITY;
      if (r == 0) out_hit[q] = (i >= 0 && b >= tau) ? 1 : 0;
    }
    if (i < 0) {  // the cache is exhausted: the remaining positions are empty
      for (int rr = r + 1 + tid; rr < k; rr += 1024) {
        out_idx[(long)q * k + rr] = -1;
        out_score[(long)q * k + rr] = -INFINITY;
      }
      break;
    }
    ps = b;
    pj = i;
    if (REG && (i & 1023) == tid) taken |= 1u << (unsigned)(i >> 10);
  }
}

struct BatchWs {
  float* part_dot;
  float* part_cc;
  float* scores;
  size_t bytes;
};

BatchWs carve_batch(long N, int d, int Qc, void* base) {
  BatchWs w;
  const BatchPlan p = plan_batch(N, d);
  const int QP = Qc > 16 ? 32 : 16;
  const long rows = p.tiles > 0 ? (long)p.tiles * kBR : kBR;  // padded to whole row tiles
  const BytePtr b(base);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    void* r = b + off;
    off += align_up(bytes, 256);
    return r;
  };
  w.part_dot = (float*)take((size_t)p.KS * rows * QP * 4);
  w.part_cc = (float*)take((size_t)p.KS * rows * 4);
  w.scores = (float*)take((size_t)32 * rows * 4);
  w.bytes = off;
  return w;
}

}  // namespace
}  // namespace chorus

using namespace chorus;

extern "C" {

size_t chorus_cache_lookup_batch_workspace_bytes(int64_t N, int32_t d, int32_t Q) {
  if (N < 0 || d <= 0 || Q < 0) return 0;
  return carve_batch((long)N, d, Q > 32 ? 32 : Q, nullptr).bytes;
}

int32_t chorus_cache_lookup_batch(const float* cache_emb, int64_t N, int32_t d, const float* queries, int32_t Q, float tau,
                                  int32_t k, int32_t* out_index, float* out_score, int32_t* out_hit, void* ws,
                                  size_t ws_bytes, void* stream) {
  if (N < 0 || d <= 0 || Q < 0 || k < 1 || k > 1024) return CHORUS_E_ARG;
  if (Q == 0) return CHORUS_OK;
  if (!queries || !out_index || !out_score || !out_hit || (N > 0 && !cache_emb)) return CHORUS_E_ARG;
  if ((d & 3) != 0) return CHORUS_E_SHAPE;
  if (!aligned16(cache_emb) || !aligned16(queries)) return CHORUS_E_ARG;
  if (N > 0x7fffff00LL) return CHORUS_E_SHAPE;
  if (!ws || !aligned16(ws) || ws_bytes < chorus_cache_lookup_batch_workspace_bytes(N, d, Q)) return CHORUS_E_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const BatchPlan p = plan_batch((long)N, d);
  for (int q0 = 0; q0 < Q; q0 += 32) {
    const int Qc = Q - q0 < 32 ? Q - q0 : 32;
    const int QP = Qc > 16 ? 32 : 16;
    BatchWs w = carve_batch((long)N, d, Q > 32 ? 32 : Q, ws);
    const float* qs = queries + (long)q0 * d;
    if (N > 0) {
      dim3 grid((unsigned)p.tiles, (unsigned)p.KS);
      if (QP == 32)
        hipLaunchKernelGGL(lookup_batch_scores_kernel<2>, grid, dim3(256), 0, s, cache_emb, qs, w.part_dot, w.part_cc,
                           (long)N, d, Qc, p.chunks_per_slice);
      else
        hipLaunchKernelGGL(lookup_batch_scores_kernel<1>, grid, dim3(256), 0, s, cache_emb, qs, w.part_dot, w.part_cc,
                           (long)N, d, Qc, p.chunks_per_slice);
      CHORUS_LAUNCH_CHECK();
    }
    const long Npad = (long)p.tiles * kBR;
    if (N > 0) {
      hipLaunchKernelGGL(lookup_batch_final_kernel, dim3((unsigned)((N + 1023) / 1024), (unsigned)Qc), dim3(256), 0, s,
                         w.part_dot, w.part_cc, qs, w.scores, (long)N, Npad, d, QP, p.KS);
      CHORUS_LAUNCH_CHECK();
    }
    if (N <= 8 * 1024)
      hipLaunchKernelGGL(lookup_topk_kernel<true>, dim3(Qc), dim3(1024), 0, s, w.scores, (long)N, Npad, k, tau,
                         out_index + (long)q0 * k, out_score + (long)q0 * k, out_hit + q0);
    else
      hipLaunchKernelGGL(lookup_topk_kernel<false>, dim3(Qc), dim3(1024), 0, s, w.scores, (long)N, Npad, k, tau,
                         out_index + (long)q0 * k, out_score + (long)q0 * k, out_hit + q0);
    CHORUS_LAUNCH_CHECK();
  }
  return CHORUS_OK;
}

}  // extern "C"
