// Stage-1 retrieval: top-1 cosine similarity over the prompt-embedding cache
// (Sec. 3.1 "Full Reuse"). HBM-bound: the [N, d] fp32 cache is streamed once.
#include "common.h"

namespace chorus {

thread_local int32_t g_last_hip_error = 0;

namespace {

constexpr int kRowsPerBlock = 4;  // one wave per cache row

// One wave per row: lanes stride over the row in float4, then a butterfly
// reduction. The order of additions depends only on d, never on the row index,
// so identical rows produce identical values. The kernel stores r_j = <q, c_j> / |c_j|;
// the query norm is a positive constant for the whole scan and is applied once, in the
// argmax kernel (score_j = r_j / |q|), which keeps this HBM-bound loop at 8 FMAs per
// 16 bytes read.
__global__ __launch_bounds__(256) void lookup_scores_kernel(const float* __restrict__ cache,
                                                            const float* __restrict__ query, float* __restrict__ scores,
                                                            long N, int d) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (row >= N) return;
  const float4* c4 = reinterpret_cast<const float4*>(cache + row * (long)d);
  const float4* q4 = reinterpret_cast<const float4*>(query);
  const int n4 = d >> 2;
  float dot = 0.f, cc = 0.f;
  int i = lane;
  // 8 independent 16-byte loads in flight per lane
  for (; i + 7 * 64 < n4; i += 8 * 64) {
    float4 c[8], q[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) c[u] = ld_stream_f4(&c4[i + u * 64]);
#pragma unroll
    for (int u = 0; u < 8; ++u) q[u] = q4[i + u * 64];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      dot += c[u].x * q[u].x + c[u].y * q[u].y + c[u].z * q[u].z + c[u].w * q[u].w;
      cc += c[u].x * c[u].x + c[u].y * c[u].y + c[u].z * c[u].z + c[u].w * c[u].w;
    }
  }
  for (; i < n4; i += 64) {
    float4 c = ld_stream_f4(&c4[i]);
    float4 q = q4[i];
    dot += c.x * q.x + c.y * q.y + c.z * q.z + c.w * q.w;
    cc += c.x * c.x + c.y * c.y + c.z * c.z + c.w * c.w;
  }
  dot = wave_sum(dot);
  cc = wave_sum(cc);
  if (lane == 0) {
    float nc = sqrtf(cc);
    float s = nc > 0.f ? dot / nc : -INFINITY;
    if (!(s == s)) s = -INFINITY;
    scores[row] = s;
  }
}

// Single workgroup: |q|, then max score with the lowest index among equal maxima.
__global__ __launch_bounds__(1024) void lookup_argmax_kernel(const float* __restrict__ scores, long N,
                                                             const float* __restrict__ query, int d, float tau,
                                                             chorus_lookup_result* __restrict__ out) {
  __shared__ float sv[16];
  __shared__ long si[16];
  __shared__ float sq[16];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nw = blockDim.x >> 6;
  float qq = 0.f;
  for (int i = threadIdx.x; i < d; i += blockDim.x) qq += query[i] * query[i];
  qq = wave_sum(qq);
  float best = -INFINITY;
  long bi = N > 0 ? N : -1;  // sentinel larger than any index
  for (long j = threadIdx.x; j < N; j += blockDim.x) {
    float s = scores[j];
    if (s > best || (s == best && j < bi)) {
      best = s;
      bi = j;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ob = __shfl_xor(best, o, 64);
    long oi = __shfl_xor(bi, o, 64);
    if (ob > best || (ob == best && oi < bi)) {
      best = ob;
      bi = oi;
    }
  }
  if (lane == 0) {
    sv[wave] = best;
    si[wave] = bi;
    sq[wave] = qq;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float qsum = 0.f;
    for (int w = 0; w < nw; ++w) qsum += sq[w];
    for (int w = 1; w < nw; ++w) {
      if (sv[w] > best || (sv[w] == best && si[w] < bi)) {
        best = sv[w];
        bi = si[w];
      }
    }
    chorus_lookup_result r;
    if (N <= 0) {
      r.index = -1;
      r.score = -INFINITY;
      r.hit = 0;
    } else {
      const float nq = sqrtf(qsum);
      float m = (nq > 0.f && best > -INFINITY) ? best / nq : -INFINITY;
      if (!(m == m)) m = -INFINITY;
      // every score -inf (zero-norm query or rows): index 0, like a first-maximum scan
      r.index = (int32_t)((bi >= N || m == -INFINITY) ? 0 : bi);
      r.score = m;
      r.hit = m >= tau ? 1 : 0;
    }
    *out = r;
  }
}

}  // namespace
}  // namespace chorus

using namespace chorus;

extern "C" {

int32_t chorus_version(void) { return 100; }
int32_t chorus_last_hip_error(void) { return g_last_hip_error; }

size_t chorus_cache_lookup_workspace_bytes(int64_t N) { return align_up((size_t)(N > 0 ? N : 1) * sizeof(float), 256); }

int32_t chorus_cache_lookup(const float* cache_emb, int64_t N, int32_t d, const float* query, float tau,
                            chorus_lookup_result* out, void* ws, size_t ws_bytes, void* stream) {
  if (N < 0 || d <= 0 || !out || !query) return CHORUS_E_ARG;
  if (N > 0 && !cache_emb) return CHORUS_E_ARG;
  if ((d & 3) != 0) return CHORUS_E_SHAPE;
  if (!aligned16(cache_emb) || !aligned16(query)) return CHORUS_E_ARG;
  if (!ws || ws_bytes < chorus_cache_lookup_workspace_bytes(N)) return CHORUS_E_WORKSPACE;
  if (N > (int64_t)kRowsPerBlock * 0x7fffffffLL) return CHORUS_E_SHAPE;
  hipStream_t s = (hipStream_t)stream;
  float* scores = (float*)ws;
  if (N > 0) {
    unsigned grid = (unsigned)((N + kRowsPerBlock - 1) / kRowsPerBlock);
    hipLaunchKernelGGL(lookup_scores_kernel, dim3(grid), dim3(256), 0, s, cache_emb, query, scores, (long)N, d);
    CHORUS_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(lookup_argmax_kernel, dim3(1), dim3(1024), 0, s, scores, (long)N, query, d, tau, out);
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

}  // extern "C"
