// Stage-1 retrieval over a low-precision copy of the prompt-embedding cache (cache maintenance around
// Sec. 3.1 "Full Reuse"): the scan reads bf16 (half the bytes) or FP8 E4M3 rows (a quarter), and the rows whose
// approximate score lies within a proven margin of the best one are re-scored from the fp32 rows, so the result
// is the fp32 lookup's. HBM-bound like the fp32 scan.
//
// Why the margin suffices: replacing a row c by its low-precision copy c^ turns it by at most
// asin(|c^ - c| / |c|), and a cosine moves by at most that angle. bf16 keeps 8 significant bits (every element
// within 2^-8 of itself); FP8 E4M3 keeps 4 down to 2^-6 and steps of 2^-9 below, on a row scaled so that its
// largest magnitude is 448. With eps that bound, the true best row's approximate score is within 2 eps of the
// best approximate score.
#include <cmath>

#include "chorus_ops.h"
#include "common.h"
#include "lookup_row.h"

namespace chorus {
namespace {

constexpr int kWaves = 4;             // waves per workgroup of the scan, one row per wave at a time
constexpr int kMaxScanBlocks = 4096;
constexpr size_t kHeaderBytes = 256;  // |q|^2

inline long scan_blocks(long N) {
  long g = (N + kWaves - 1) / kWaves;
  return g < kMaxScanBlocks ? g : kMaxScanBlocks;
}

struct RerankPartial;
struct LpWs {
  float* qnorm2;
  float* partial_max;      // [scan_blocks]
  RerankPartial* rerank;   // [scan_blocks]
  float* scores;           // [N] approximate r_j = <q, c^_j> / |c^_j|
  size_t bytes;
};
LpWs carve_lp(long N, void* base) {
  const BytePtr p(base);
  LpWs w;
  size_t off = 0;
  w.qnorm2 = (float*)(p + off);
  off += kHeaderBytes;
  w.partial_max = (float*)(p + off);
  off += align_up((size_t)kMaxScanBlocks * sizeof(float), 256);
  w.rerank = (RerankPartial*)(p + off);
  off += (size_t)kMaxScanBlocks * 16;
  w.scores = (float*)(p + off);
  off += align_up((size_t)(N > 0 ? N : 1) * sizeof(float), 256);
  w.bytes = off;
  return w;
}

// ---- decoding 16 bytes of a row into floats ------------------------------------------------
template <int FMT>
struct Codes;
template <>
struct Codes<CHORUS_LP_BF16> {
  static constexpr int kPer16 = 8;  // elements per 16-byte load
  __device__ static __forceinline__ void decode(const u32x4& v, float (&f)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(v[i] << 16);
      f[2 * i + 1] = __uint_as_float(v[i] & 0xffff0000u);
    }
  }
};
template <>
struct Codes<CHORUS_LP_FP8> {
  static constexpr int kPer16 = 16;
  __device__ static __forceinline__ void decode(const u32x4& v, float (&f)[16]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const auto lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)v[i], false);  // bytes 0, 1
      const auto hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)v[i], true);   // bytes 2, 3
      f[4 * i] = lo[0];
      f[4 * i + 1] = lo[1];
      f[4 * i + 2] = hi[0];
      f[4 * i + 3] = hi[1];
    }
  }
};

// ---- store: fp32 rows -> low-precision rows ---------------------------------------------------
// One wave per row. bf16: round to nearest even. FP8: y = c * (448 / max|c|), both single fp32 operations,
// clamped to [-448, 448] (a product may land one fp32 step above 448), then rounded to nearest even.
template <int FMT>
__global__ __launch_bounds__(256) void lowprec_store_kernel(const float* __restrict__ emb, long n_rows, int d,
                                                            void* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n_rows) return;
  const float4* c4 = reinterpret_cast<const float4*>(emb + row * (long)d);
  const int n4 = d >> 2;
  if (FMT == CHORUS_LP_BF16) {
    uint2* o = reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(out) + row * (long)d);
    for (int i = lane; i < n4; i += 64) {
      const float4 c = c4[i];
      uint2 w;
      w.x = pack_bf16x2(c.x, c.y);
      w.y = pack_bf16x2(c.z, c.w);
      o[i] = w;
    }
  } else {
    float amax = 0.f;
    for (int i = lane; i < n4; i += 64) {
      const float4 c = c4[i];
      amax = fmaxf(fmaxf(amax, fmaxf(fabsf(c.x), fabsf(c.y))), fmaxf(fabsf(c.z), fabsf(c.w)));
    }
    amax = wave_max(amax);
    const float inv = amax > 0.f ? __fdiv_rn(448.0f, amax) : 0.f;
    uint32_t* o = reinterpret_cast<uint32_t*>(reinterpret_cast<uint8_t*>(out) + row * (long)d);
    for (int i = lane; i < n4; i += 64) {
      const float4 c = c4[i];
      const float y0 = fminf(fmaxf(__fmul_rn(c.x, inv), -448.f), 448.f), y1 = fminf(fmaxf(__fmul_rn(c.y, inv), -448.f), 448.f);
      const float y2 = fminf(fmaxf(__fmul_rn(c.z, inv), -448.f), 448.f), y3 = fminf(fmaxf(__fmul_rn(c.w, inv), -448.f), 448.f);
      int w = __builtin_amdgcn_cvt_pk_fp8_f32(y0, y1, 0, false);
      w = __builtin_amdgcn_cvt_pk_fp8_f32(y2, y3, w, true);
      o[i] = (uint32_t)w;
    }
  }
}

// ---- scan of the low-precision rows -------------------------------------------------------------
template <int FMT>
__global__ __launch_bounds__(kWaves * 64) void lowprec_scan_kernel(const void* __restrict__ cache_lp,
                                                                   const float* __restrict__ query, long N, int d,
                                                                   float* __restrict__ scores,
                                                                   float* __restrict__ partial_max,
                                                                   float* __restrict__ qnorm2) {
  constexpr int E = Codes<FMT>::kPer16;
  constexpr int U = 4;  // 16-byte loads in flight per lane
  __shared__ float sv[kWaves];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n16 = d / E;  // 16-byte chunks per row
  const long row_bytes = (long)d * (16 / E);
  float best = -INFINITY;
  const long stride = (long)gridDim.x * kWaves;
  for (long row = (long)blockIdx.x * kWaves + wave; row < N; row += stride) {
    const u32x4* c16 = reinterpret_cast<const u32x4*>(reinterpret_cast<const uint8_t*>(cache_lp) + row * row_bytes);
    float dot = 0.f, cc = 0.f;
    int i = lane;
    for (; i + (U - 1) * 64 < n16; i += U * 64) {
      u32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(&c16[i + u * 64]);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float f[E];
        Codes<FMT>::decode(v[u], f);
        const float4* q4 = reinterpret_cast<const float4*>(query + (long)(i + u * 64) * E);
#pragma unroll
        for (int e4 = 0; e4 < E / 4; ++e4) {
          const float4 q = q4[e4];
          dot += f[4 * e4] * q.x + f[4 * e4 + 1] * q.y + f[4 * e4 + 2] * q.z + f[4 * e4 + 3] * q.w;
          cc += f[4 * e4] * f[4 * e4] + f[4 * e4 + 1] * f[4 * e4 + 1] + f[4 * e4 + 2] * f[4 * e4 + 2] + f[4 * e4 + 3] * f[4 * e4 + 3];
        }
      }
    }
    for (; i < n16; i += 64) {
      const u32x4 v = __builtin_nontemporal_load(&c16[i]);
      float f[E];
      Codes<FMT>::decode(v, f);
      const float4* q4 = reinterpret_cast<const float4*>(query + (long)i * E);
#pragma unroll
      for (int e4 = 0; e4 < E / 4; ++e4) {
        const float4 q = q4[e4];
        dot += f[4 * e4] * q.x + f[4 * e4 + 1] * q.y + f[4 * e4 + 2] * q.z + f[4 * e4 + 3] * q.w;
        cc += f[4 * e4] * f[4 * e4] + f[4 * e4 + 1] * f[4 * e4 + 1] + f[4 * e4 + 2] * f[4 * e4 + 2] + f[4 * e4 + 3] * f[4 * e4 + 3];
      }
    }
    dot = wave_sum(dot);
    cc = wave_sum(cc);
    const float r = row_ratio(dot, cc);
    if (lane == 0) scores[row] = r;
    best = fmaxf(best, r);
  }
  if (blockIdx.x == 0 && wave == 0) {  // |q|^2 exactly as the fp32 lookup sums it
    float qq = 0.f;
    const float4* q4 = reinterpret_cast<const float4*>(query);
    const int n4 = d >> 2;
    int i = lane;
    for (; i + 7 * 64 < n4; i += 8 * 64) {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float4 q = q4[i + u * 64];
        qq += q.x * q.x + q.y * q.y + q.z * q.z + q.w * q.w;
      }
    }
    for (; i < n4; i += 64) {
      const float4 q = q4[i];
      qq += q.x * q.x + q.y * q.y + q.z * q.z + q.w * q.w;
    }
    qq = wave_sum(qq);
    if (lane == 0) *qnorm2 = qq;
  }
  if (lane == 0) sv[wave] = best;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kWaves; ++w) best = fmaxf(best, sv[w]);
    partial_max[blockIdx.x] = best;
  }
}

// ---- candidates and exact re-rank ---------------------------------------------------------------
// threshold = best approximate r - margin * |q| (r = cosine * |q|); every row at or above it is re-scored from its
// fp32 row by a whole wave with the fp32 lookup's own row pass. The launch has the scan's shape (one wave per row at
// a time), so even when every row is a candidate (FP8 on a query far from every entry) the re-rank costs one fp32
// scan, spread over the chip; usually a single wave has work. Each wave first reduces the scan's partial maxima
// itself (at most 4096 floats, L2-resident).
struct RerankPartial {
  float r;
  int32_t idx;
  int32_t count;
  int32_t pad;
};
static_assert(sizeof(RerankPartial) == 16, "workspace carving assumes 16 bytes per partial");

__global__ __launch_bounds__(kWaves * 64) void lowprec_rerank_kernel(const float* __restrict__ cache_emb,
                                                                     const float* __restrict__ query, long N, int d,
                                                                     const float* __restrict__ scores,
                                                                     const float* __restrict__ partial_max, int nparts,
                                                                     const float* __restrict__ qnorm2, float margin,
                                                                     RerankPartial* __restrict__ partial) {
  __shared__ float sv[kWaves];
  __shared__ int32_t si[kWaves];
  __shared__ int32_t sc[kWaves];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float mx = -INFINITY;
  for (int j = lane; j < nparts; j += 64) mx = fmaxf(mx, partial_max[j]);
  mx = wave_max(mx);
  const float nq = sqrtf(*qnorm2);
  // no finite score (all rows zero) or a zero query: every exact score is -inf as well, nothing is re-scored
  const float thr = nq > 0.f ? mx - margin * nq : -INFINITY;
  const float4* q4 = reinterpret_cast<const float4*>(query);
  const int n4 = d >> 2;
  float best = -INFINITY;
  int32_t bi = 0x7fffffff, count = 0;
  const long stride = (long)gridDim.x * kWaves;
  if (thr > -INFINITY) {
    for (long row = (long)blockIdx.x * kWaves + wave; row < N; row += stride) {
      if (!(scores[row] >= thr)) continue;  // one address per wave: uniform
      float dot, cc, qq;
      fp32_row_products(reinterpret_cast<const float4*>(cache_emb + row * (long)d), q4, n4, lane, dot, cc, qq);
      const float r = row_ratio(dot, cc);
      ++count;
      if (r > best) {  // rows ascend within a wave
        best = r;
        bi = (int32_t)row;
      }
    }
  }
  if (lane == 0) {
    sv[wave] = best;
    si[wave] = bi;
    sc[wave] = count;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
      if (sv[w] > best || (sv[w] == best && si[w] < bi)) {
        best = sv[w];
        bi = si[w];
      }
      count += sc[w];
    }
    RerankPartial p;
    p.r = best;
    p.idx = bi;
    p.count = count;
    p.pad = 0;
    partial[blockIdx.x] = p;
  }
}

// Single workgroup: the best exact r among the workgroup partials (lowest index among equal ones), the number of
// re-scored rows, then the division by |q| and the threshold test, as in the fp32 lookup.
__global__ __launch_bounds__(256) void lowprec_final_kernel(const RerankPartial* __restrict__ partial, int nparts,
                                                            const float* __restrict__ qnorm2, long N, float tau,
                                                            chorus_lookup_result* __restrict__ out,
                                                            int32_t* __restrict__ n_rescored) {
  __shared__ float sv[4];
  __shared__ int32_t si[4];
  __shared__ int32_t sc[4];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float best = -INFINITY;
  int32_t bi = 0x7fffffff, count = 0;
  for (int j = threadIdx.x; j < nparts; j += 256) {
    const RerankPartial p = partial[j];
    count += p.count;
    if (p.r > best || (p.r == best && p.idx < bi)) {
      best = p.r;
      bi = p.idx;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ob = __shfl_xor(best, o, 64);
    const int32_t oi = __shfl_xor(bi, o, 64);
    count += __shfl_xor(count, o, 64);
    if (ob > best || (ob == best && oi < bi)) {
      best = ob;
      bi = oi;
    }
  }
  if (lane == 0) {
    sv[wave] = best;
    si[wave] = bi;
    sc[wave] = count;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) {
      if (sv[w] > best || (sv[w] == best && si[w] < bi)) {
        best = sv[w];
        bi = si[w];
      }
      count += sc[w];
    }
    chorus_lookup_result r;
    if (N <= 0) {
      r.index = -1;
      r.score = -INFINITY;
      r.hit = 0;
    } else {
      const float nq = sqrtf(*qnorm2);
      float mm = (nq > 0.f && best > -INFINITY) ? best / nq : -INFINITY;
      if (!(mm == mm)) mm = -INFINITY;
      r.index = (bi == 0x7fffffff || mm == -INFINITY) ? 0 : bi;
      r.score = mm;
      r.hit = mm >= tau ? 1 : 0;
    }
    *out = r;
    if (n_rescored) *n_rescored = count;
  }
}

inline double lowprec_margin(int format, int d) {
  const double delta = format == CHORUS_LP_BF16 ? std::ldexp(1.0, -8)
                                                 : std::ldexp(1.0, -4) + std::sqrt((double)d) * std::ldexp(1.0, -10) / 448.0;
  // twice the bound, plus room for the fp32 summation of the approximate scores themselves
  return 2.0 * std::asin(delta) + 4.0e-6 * std::sqrt((double)d);
}

}  // namespace
}  // namespace chorus

using namespace chorus;

extern "C" {

size_t chorus_cache_lowprec_bytes(int64_t N, int32_t d, int32_t format) {
  if (N < 0 || d <= 0 || (format != CHORUS_LP_BF16 && format != CHORUS_LP_FP8)) return 0;
  return (size_t)N * (size_t)d * (format == CHORUS_LP_BF16 ? 2 : 1);
}

int32_t chorus_cache_lowprec_store(const float* emb, int64_t n_rows, int32_t d, int32_t format, void* out, void* stream) {
  if (n_rows < 0 || d <= 0) return CHORUS_E_ARG;
  if (format != CHORUS_LP_BF16 && format != CHORUS_LP_FP8) return CHORUS_E_ARG;
  if (n_rows == 0) return CHORUS_OK;
  if (!emb || !out) return CHORUS_E_ARG;
  if (d % 16) return CHORUS_E_SHAPE;
  if (!aligned16(emb) || !aligned16(out)) return CHORUS_E_ARG;
  if ((n_rows + 3) / 4 > 0x7fffffffLL) return CHORUS_E_SHAPE;
  const unsigned grid = (unsigned)((n_rows + 3) / 4);
  hipStream_t s = (hipStream_t)stream;
  if (format == CHORUS_LP_BF16)
    hipLaunchKernelGGL(lowprec_store_kernel<CHORUS_LP_BF16>, dim3(grid), dim3(256), 0, s, emb, (long)n_rows, d, out);
  else
    hipLaunchKernelGGL(lowprec_store_kernel<CHORUS_LP_FP8>, dim3(grid), dim3(256), 0, s, emb, (long)n_rows, d, out);
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

size_t chorus_cache_lookup_lowprec_workspace_bytes(int64_t N) { return carve_lp(N > 0 ? (long)N : 0, nullptr).bytes; }

int32_t chorus_cache_lookup_lowprec(const float* cache_emb, const void* cache_lp, int32_t format, int64_t N, int32_t d,
                                    const float* query, float tau, chorus_lookup_result* out, int32_t* n_rescored, void* ws,
                                    size_t ws_bytes, void* stream) {
  if (N < 0 || d <= 0 || !out || !query) return CHORUS_E_ARG;
  if (format != CHORUS_LP_BF16 && format != CHORUS_LP_FP8) return CHORUS_E_ARG;
  if (N > 0 && (!cache_emb || !cache_lp)) return CHORUS_E_ARG;
  if (d % 16) return CHORUS_E_SHAPE;
  if (N > 0x7fffffffLL - 1) return CHORUS_E_SHAPE;
  if (!aligned16(cache_emb) || !aligned16(cache_lp) || !aligned16(query) || !aligned16(ws)) return CHORUS_E_ARG;
  if (!ws || ws_bytes < chorus_cache_lookup_lowprec_workspace_bytes(N)) return CHORUS_E_WORKSPACE;
  LpWs w = carve_lp((long)N, ws);
  hipStream_t s = (hipStream_t)stream;
  int nparts = 0;
  if (N > 0) {
    nparts = (int)scan_blocks((long)N);
    if (format == CHORUS_LP_BF16)
      hipLaunchKernelGGL(lowprec_scan_kernel<CHORUS_LP_BF16>, dim3((unsigned)nparts), dim3(kWaves * 64), 0, s, cache_lp, query,
                         (long)N, d, w.scores, w.partial_max, w.qnorm2);
    else
      hipLaunchKernelGGL(lowprec_scan_kernel<CHORUS_LP_FP8>, dim3((unsigned)nparts), dim3(kWaves * 64), 0, s, cache_lp, query,
                         (long)N, d, w.scores, w.partial_max, w.qnorm2);
    CHORUS_LAUNCH_CHECK();
  }
  if (N > 0) {
    hipLaunchKernelGGL(lowprec_rerank_kernel, dim3((unsigned)nparts), dim3(kWaves * 64), 0, s, cache_emb, query, (long)N, d,
                       w.scores, w.partial_max, nparts, w.qnorm2, (float)lowprec_margin(format, d), w.rerank);
    CHORUS_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(lowprec_final_kernel, dim3(1), dim3(256), 0, s, w.rerank, nparts, w.qnorm2, (long)N, tau, out, n_rescored);
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

}  // extern "C"
