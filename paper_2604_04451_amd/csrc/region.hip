// Selective region path (Sec. 3.3): mask -> ascending token list, row gather /
// scatter, and the latent fusion of Eq. 6. All integer / bit-copy work, HBM-bound.
#include "common.h"

namespace chorus {
namespace {

constexpr int kCompactThreads = 256;
constexpr int kBytesPerThread = 16;
constexpr int kCompactTile = kCompactThreads * kBytesPerThread;  // mask bytes per workgroup

__device__ __forceinline__ uint32_t nonzero_bits16(const uint8_t* __restrict__ mask, long base, long L) {
  uint32_t bits = 0;
  if (base + kBytesPerThread <= L && ((reinterpret_cast<uintptr_t>(mask + base) & 15u) == 0)) {
    uint4 v = *reinterpret_cast<const uint4*>(mask + base);
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int b = 0; b < 4; ++b)
        if ((w[k] >> (8 * b)) & 0xffu) bits |= 1u << (4 * k + b);
  } else {
    for (int b = 0; b < kBytesPerThread; ++b)
      if (base + b < L && mask[base + b]) bits |= 1u << b;
  }
  return bits;
}

// exclusive scan of one int per thread over a 256-thread workgroup; returns the
// thread's offset and, in *total, the workgroup sum
__device__ __forceinline__ int block_exclusive_scan(int v, int* total) {
  __shared__ int wsum[kCompactThreads / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int t = __shfl_up(inc, o, 64);
    if (lane >= o) inc += t;
  }
  if (lane == 63) wsum[wave] = inc;
  __syncthreads();
  int off = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kCompactThreads / 64; ++w) {
    if (w < wave) off += wsum[w];
    tot += wsum[w];
  }
  *total = tot;
  return off + inc - v;
}

__global__ __launch_bounds__(kCompactThreads) void compact_count_kernel(const uint8_t* __restrict__ mask, long L,
                                                                        int* __restrict__ tile_counts) {
  long base = (long)blockIdx.x * kCompactTile + (long)threadIdx.x * kBytesPerThread;
  int c = __popc(nonzero_bits16(mask, base, L));
  int total;
  block_exclusive_scan(c, &total);
  if (threadIdx.x == 0) tile_counts[blockIdx.x] = total;
}

// single workgroup: exclusive scan of the per-tile counts, in place; writes the grand total
__global__ __launch_bounds__(kCompactThreads) void compact_scan_kernel(int* __restrict__ tile_counts, int ntiles,
                                                                       int* __restrict__ count_out) {
  __shared__ int carry_s;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  for (int base = 0; base < ntiles; base += kCompactThreads) {
    int i = base + threadIdx.x;
    int v = i < ntiles ? tile_counts[i] : 0;
    int total;
    int off = block_exclusive_scan(v, &total);
    int carry = carry_s;
    if (i < ntiles) tile_counts[i] = carry + off;
    __syncthreads();
    if (threadIdx.x == 0) carry_s = carry + total;
    __syncthreads();
  }
  if (threadIdx.x == 0) *count_out = carry_s;
}

__global__ __launch_bounds__(kCompactThreads) void compact_write_kernel(const uint8_t* __restrict__ mask, long L,
                                                                        const int* __restrict__ tile_offsets,
                                                                        int* __restrict__ idx_out) {
  long base = (long)blockIdx.x * kCompactTile + (long)threadIdx.x * kBytesPerThread;
  uint32_t bits = nonzero_bits16(mask, base, L);
  int total;
  int off = block_exclusive_scan(__popc(bits), &total) + tile_offsets[blockIdx.x];
  while (bits) {
    int b = __ffs(bits) - 1;
    bits &= bits - 1;
    idx_out[off++] = (int)(base + b);
  }
}

template <typename V, bool SCATTER>
__global__ __launch_bounds__(256) void move_rows_kernel(V* __restrict__ dst, const V* __restrict__ src,
                                                        const int* __restrict__ idx, long Ls, int vec_per_row) {
  long total = Ls * vec_per_row;
  for (long g = (long)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += (long)gridDim.x * blockDim.x) {
    long i = g / vec_per_row;
    int c = (int)(g - i * vec_per_row);
    long r = idx[i];
    if (SCATTER)
      dst[r * vec_per_row + c] = src[g];
    else
      dst[g] = src[r * vec_per_row + c];
  }
}

// Eq. 6 as a select. A thread owns kBlendU float4 (along W) spaced a grid apart and issues
// all their loads before any store; the source that is not selected is not read unless the
// four elements straddle tokens that disagree.
constexpr int kBlendU = 4;

template <int PW>  // PW > 0: patch width known at compile time (1, 2 or 4); 0: runtime pw
__global__ __launch_bounds__(256) void blend_vec4_kernel(float4* out, const float4* Lc, const float4* SL,  // out may alias a source
                                                         const uint8_t* __restrict__ mask, unsigned nvec, unsigned T,
                                                         unsigned H, unsigned W4, unsigned ph, unsigned pw,
                                                         unsigned Hm, unsigned Wm) {
  // 32-bit index arithmetic on purpose: 64-bit divisions cost more than the memory traffic here
  const unsigned stride = gridDim.x * blockDim.x;
  const unsigned v0 = blockIdx.x * blockDim.x + threadIdx.x;
  f32x4 a[kBlendU], b[kBlendU];  // native vectors: arrays of HIP's float4 struct would live in scratch memory
  int sel[kBlendU];  // bit e set: element e keeps L; -1: out of range
#pragma unroll
  for (int u = 0; u < kBlendU; ++u) {
    const unsigned v = v0 + u * stride;
    sel[u] = -1;
    if (v >= nvec) continue;
    const unsigned row = v / W4;
    const unsigned x4 = v - row * W4;
    const unsigned rt = row / H;
    const unsigned y = row - rt * H;
    const unsigned t = rt % T;
    const uint8_t* mrow = mask + (t * Hm + y / ph) * Wm;
    const unsigned x = x4 * 4;
    int m = 0;
    if (PW == 2) {
      m = (mrow[x >> 1] != 0 ? 3 : 0) | (mrow[(x >> 1) + 1] != 0 ? 12 : 0);
    } else if (PW == 4) {
      m = mrow[x >> 2] != 0 ? 15 : 0;
    } else if (PW == 1) {
#pragma unroll
      for (int e = 0; e < 4; ++e) m |= (mrow[x + e] != 0) << e;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) m |= (mrow[(x + e) / pw] != 0) << e;
    }
    sel[u] = m;
  }
  // all mask bytes are requested before the first data load depends on one of them
#pragma unroll
  for (int u = 0; u < kBlendU; ++u) {
    const unsigned v = v0 + u * stride;
    if (sel[u] < 0) continue;
    if (sel[u] != 0) a[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(&Lc[v]));
    if (sel[u] != 15) b[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(&SL[v]));
  }
#pragma unroll
  for (int u = 0; u < kBlendU; ++u) {
    if (sel[u] < 0) continue;
    const unsigned v = v0 + u * stride;
    const int m = sel[u];
    f32x4 r;
    if (m == 15) {
      r = a[u];
    } else if (m == 0) {
      r = b[u];
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) r[e] = ((m >> e) & 1) ? a[u][e] : b[u][e];
    }
    __builtin_nontemporal_store(r, reinterpret_cast<f32x4*>(&out[v]));
  }
}

__global__ __launch_bounds__(256) void blend_scalar_kernel(float* out, const float* Lc, const float* SL,
                                                          
                                                           const uint8_t* __restrict__ mask, long n, int T, int H,
                                                           int W, int ph, int pw, int Hm, int Wm) {
  long v = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (v >= n) return;
  int x = (int)(v % W);
  long row = v / W;
  int y = (int)(row % H);
  int t = (int)((row / H) % T);
  bool m = mask[((long)t * Hm + y / ph) * Wm + x / pw] != 0;
  out[v] = m ? Lc[v] : SL[v];
}

}  // namespace
}  // namespace chorus

using namespace chorus;

extern "C" {

size_t chorus_region_compact_workspace_bytes(int64_t L) {
  int64_t ntiles = L > 0 ? (L + kCompactTile - 1) / kCompactTile : 1;
  return align_up((size_t)ntiles * sizeof(int), 256);
}

int32_t chorus_region_compact(const uint8_t* mask, int64_t L, int32_t* idx_out, int32_t* count_out, void* ws,
                              size_t ws_bytes, void* stream) {
  if (L < 0 || !count_out) return CHORUS_E_ARG;
  if (L > 0 && (!mask || !idx_out)) return CHORUS_E_ARG;
  if (L > 0x7fffffffLL) return CHORUS_E_SHAPE;
  if (!ws || ws_bytes < chorus_region_compact_workspace_bytes(L)) return CHORUS_E_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  int* tiles = (int*)ws;
  int ntiles = (int)((L + kCompactTile - 1) / kCompactTile);
  if (ntiles > 0) {
    hipLaunchKernelGGL(compact_count_kernel, dim3(ntiles), dim3(kCompactThreads), 0, s, mask, (long)L, tiles);
    CHORUS_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(compact_scan_kernel, dim3(1), dim3(kCompactThreads), 0, s, tiles, ntiles, count_out);
  CHORUS_LAUNCH_CHECK();
  if (ntiles > 0) {
    hipLaunchKernelGGL(compact_write_kernel, dim3(ntiles), dim3(kCompactThreads), 0, s, mask, (long)L, tiles, idx_out);
    CHORUS_LAUNCH_CHECK();
  }
  return CHORUS_OK;
}

static int32_t move_rows(void* dst, const void* src, const int32_t* idx, int64_t Ls, int64_t row_bytes, void* stream,
                         bool scatter) {
  if (Ls < 0 || row_bytes <= 0) return CHORUS_E_ARG;
  if (Ls == 0) return CHORUS_OK;
  if (!dst || !src || !idx) return CHORUS_E_ARG;
  if (row_bytes & 3) return CHORUS_E_SHAPE;
  hipStream_t s = (hipStream_t)stream;
  bool v16 = (row_bytes % 16 == 0) && aligned16(dst) && aligned16(src);
  int64_t vpr = v16 ? row_bytes / 16 : row_bytes / 4;
  if (vpr > 0x7fffffffLL) return CHORUS_E_SHAPE;
  int64_t total = Ls * vpr;
  unsigned grid = (unsigned)((total + 255) / 256 < 65536 * 16 ? (total + 255) / 256 : 65536 * 16);
  if (v16) {
    if (scatter)
      hipLaunchKernelGGL((move_rows_kernel<uint4, true>), dim3(grid), dim3(256), 0, s, (uint4*)dst, (const uint4*)src,
                         idx, (long)Ls, (int)vpr);
    else
      hipLaunchKernelGGL((move_rows_kernel<uint4, false>), dim3(grid), dim3(256), 0, s, (uint4*)dst,
                         (const uint4*)src, idx, (long)Ls, (int)vpr);
  } else {
    if (scatter)
      hipLaunchKernelGGL((move_rows_kernel<uint32_t, true>), dim3(grid), dim3(256), 0, s, (uint32_t*)dst,
                         (const uint32_t*)src, idx, (long)Ls, (int)vpr);
    else
      hipLaunchKernelGGL((move_rows_kernel<uint32_t, false>), dim3(grid), dim3(256), 0, s, (uint32_t*)dst,
                         (const uint32_t*)src, idx, (long)Ls, (int)vpr);
  }
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

int32_t chorus_region_gather_rows(void* dst, const void* src, const int32_t* idx, int64_t Ls, int64_t row_bytes,
                                  void* stream) {
  return move_rows(dst, src, idx, Ls, row_bytes, stream, false);
}

int32_t chorus_region_scatter_rows(void* dst, const void* src, const int32_t* idx, int64_t Ls, int64_t row_bytes,
                                   void* stream) {
  return move_rows(dst, src, idx, Ls, row_bytes, stream, true);
}

int32_t chorus_region_blend(float* out, const float* L, const float* SL, const uint8_t* mask_edit, int32_t C, int32_t T,
                            int32_t H, int32_t W, int32_t ph, int32_t pw, void* stream) {
  if (C < 0 || T < 0 || H < 0 || W < 0 || ph <= 0 || pw <= 0) return CHORUS_E_ARG;
  if (H % ph || W % pw) return CHORUS_E_SHAPE;
  int64_t n = (int64_t)C * T * H * W;
  if (n == 0) return CHORUS_OK;
  if (!out || !L || !SL || !mask_edit) return CHORUS_E_ARG;
  hipStream_t s = (hipStream_t)stream;
  int Hm = H / ph, Wm = W / pw;
  if (W % 4 == 0 && aligned16(out) && aligned16(L) && aligned16(SL)) {
    int64_t nvec = n / 4;
    const int64_t per_block = 256 * kBlendU;
    if (nvec + per_block * 2 > 0x7fffffffLL) return CHORUS_E_SHAPE;  // the kernel indexes in 32 bits
    const dim3 grid((unsigned)((nvec + per_block - 1) / per_block)), block(256);
#define BLEND_LAUNCH(PWV)                                                                                        \
  hipLaunchKernelGGL(blend_vec4_kernel<PWV>, grid, block, 0, s, (float4*)out, (const float4*)L, (const float4*)SL, \
                     mask_edit, (unsigned)nvec, (unsigned)T, (unsigned)H, (unsigned)(W / 4), (unsigned)ph,        \
                     (unsigned)pw, (unsigned)Hm, (unsigned)Wm)
    if (pw == 2) BLEND_LAUNCH(2);
    else if (pw == 4) BLEND_LAUNCH(4);
    else if (pw == 1) BLEND_LAUNCH(1);
    else BLEND_LAUNCH(0);
#undef BLEND_LAUNCH
  } else {
    if ((n + 255) / 256 > 0x7fffffffLL) return CHORUS_E_SHAPE;
    hipLaunchKernelGGL(blend_scalar_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, out, L, SL, mask_edit,
                       (long)n, T, H, W, ph, pw, Hm, Wm);
  }
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

}  // extern "C"
