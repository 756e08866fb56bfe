// The fp32 row pass of the cache lookup (Sec. 3.1 "Full Reuse"), shared by the plain scan and by the re-rank of
// the low-precision scan so that a row scores the same bits in both.
#pragma once
#include "common.h"

namespace chorus {

// One wave, one cache row: dot = <q, c>, cc = <c, c>, qq = <q, q> over the n4 float4 chunks of the row, every
// lane striding over the chunks (8 independent 16-byte loads in flight per lane), then a butterfly reduction. The
// order of additions depends only on n4, never on the row, so identical rows give identical values, and qq comes
// out the same in every wave.
__device__ __forceinline__ void fp32_row_products(const float4* __restrict__ c4, const float4* __restrict__ q4, int n4,
                                                  int lane, float& dot_out, float& cc_out, float& qq_out) {
  float dot = 0.f, cc = 0.f, qq = 0.f;
  int i = lane;
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
      qq += q[u].x * q[u].x + q[u].y * q[u].y + q[u].z * q[u].z + q[u].w * q[u].w;
    }
  }
  for (; i < n4; i += 64) {
    float4 c = ld_stream_f4(&c4[i]);
    float4 q = q4[i];
    dot += c.x * q.x + c.y * q.y + c.z * q.z + c.w * q.w;
    cc += c.x * c.x + c.y * c.y + c.z * c.z + c.w * c.w;
    qq += q.x * q.x + q.y * q.y + q.z * q.z + q.w * q.w;
  }
  dot_out = wave_sum(dot);
  cc_out = wave_sum(cc);
  qq_out = wave_sum(qq);
}

// r = <q, c> / |c| (the query norm is applied once at the end of a lookup); a zero-norm row or a NaN gives -inf
__device__ __forceinline__ float row_ratio(float dot, float cc) {
  const float nc = sqrtf(cc);
  float r = nc > 0.f ? dot / nc : -INFINITY;
  if (!(r == r)) r = -INFINITY;
  return r;
}

}  // namespace chorus
