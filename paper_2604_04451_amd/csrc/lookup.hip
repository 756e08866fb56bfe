// Stage-1 retrieval: top-1 cosine similarity over the prompt-embedding cache
// (Sec. 3.1 "Full Reuse"). HBM-bound: the [N, d] fp32 cache is streamed once.
#include "common.h"
#include "lookup_row.h"

namespace chorus {

thread_local int32_t g_last_hip_error = 0;

namespace {

constexpr int kWaves = 4;            // waves per workgroup of the scan, one cache row per wave at a time
constexpr int kMaxScanBlocks = 4096; // beyond this many workgroups a wave walks several rows

// What one workgroup of the scan leaves behind: the best r_j = <q, c_j> / |c_j| among its rows and that row's
// index (the lowest one among equal values). The header in front of the partials holds |q|^2.
struct LookupPartial {
  float r;
  int32_t idx;
};
constexpr size_t kLookupHeaderBytes = 256;

inline long scan_blocks(long N) {
  long g = (N + kWaves - 1) / kWaves;
  return g < kMaxScanBlocks ? g : kMaxScanBlocks;
}
inline size_t lookup_scratch_bytes(long N) {
  return kLookupHeaderBytes + align_up((size_t)(N > 0 ? scan_blocks(N) : 1) * sizeof(LookupPartial), 256);
}

// One wave per row: lanes stride over the row in float4, then a butterfly
// reduction. The order of additions depends only on d, never on the row index,
// so identical rows produce identical values. The scan compares r_j = <q, c_j> / |c_j|;
// the query norm is a positive constant for the whole scan and is applied once, in the
// final kernel (score_j = r_j / |q|), which keeps this HBM-bound loop at 8 FMAs per
// 16 bytes read. |q|^2 falls out of the query values every wave loads anyway (the same
// additions in the same order in every wave); the first wave of the grid stores it.
__global__ __launch_bounds__(kWaves * 64) void lookup_scan_kernel(const float* __restrict__ cache,
                                                                  const float* __restrict__ query, long N, int d,
                                                                  LookupPartial* __restrict__ partial,
                                                                  float* __restrict__ qnorm2) {
  __shared__ float sv[kWaves];
  __shared__ int32_t si[kWaves];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float4* q4 = reinterpret_cast<const float4*>(query);
  const int n4 = d >> 2;
  float best = -INFINITY, qq = 0.f;
  int32_t bi = 0x7fffffff;  // larger than any index
  const long stride = (long)gridDim.x * kWaves;
  for (long row = (long)blockIdx.x * kWaves + wave; row < N; row += stride) {
    float dot, cc;
    fp32_row_products(reinterpret_cast<const float4*>(cache + row * (long)d), q4, n4, lane, dot, cc, qq);
    const float r = row_ratio(dot, cc);
    if (r > best) {  // rows ascend within a wave: a strict comparison keeps the lowest index
      best = r;
      bi = (int32_t)row;
    }
  }
  if (lane == 0) {
    sv[wave] = best;
    si[wave] = bi;
    if (blockIdx.x == 0 && wave == 0) *qnorm2 = qq;  // wave 0 of workgroup 0 always has a row
  }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
      if (sv[w] > best || (sv[w] == best && si[w] < bi)) {
        best = sv[w];
        bi = si[w];
      }
    }
    LookupPartial p;
    p.r = best;
    p.idx = bi;
    partial[blockIdx.x] = p;
  }
}

// Single workgroup: maximum over the workgroup partials with the lowest index among equal maxima, then the
// division by |q| and the threshold test.
__global__ __launch_bounds__(256) void lookup_final_kernel(const LookupPartial* __restrict__ partial, int nparts,
                                                           const float* __restrict__ qnorm2, long N, float tau,
                                                           chorus_lookup_result* __restrict__ out) {
  __shared__ float sv[4];
  __shared__ int32_t si[4];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float best = -INFINITY;
  int32_t bi = 0x7fffffff;
  for (int j = threadIdx.x; j < nparts; j += 256) {
    const LookupPartial p = partial[j];
    if (p.r > best || (p.r == best && p.idx < bi)) {
      best = p.r;
      bi = p.idx;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ob = __shfl_xor(best, o, 64);
    const int32_t oi = __shfl_xor(bi, o, 64);
    if (ob > best || (ob == best && oi < bi)) {
      best = ob;
      bi = oi;
    }
  }
  if (lane == 0) {
    sv[wave] = best;
    si[wave] = bi;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) {
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
      const float nq = sqrtf(*qnorm2);
      float m = (nq > 0.f && best > -INFINITY) ? best / nq : -INFINITY;
      if (!(m == m)) m = -INFINITY;
      // every score -inf (zero-norm query or rows): index 0, like a first-maximum scan
      r.index = (bi == 0x7fffffff || m == -INFINITY) ? 0 : bi;
      r.score = m;
      r.hit = m >= tau ? 1 : 0;
    }
    *out = r;
  }
}

// both launches of a lookup; `scratch` holds the header and the partials (lookup_scratch_bytes(N))
int32_t launch_lookup(const float* cache_emb, long N, int d, const float* query, float tau, chorus_lookup_result* out,
                      void* scratch, hipStream_t s) {
  float* qnorm2 = reinterpret_cast<float*>(scratch);
  LookupPartial* partial = reinterpret_cast<LookupPartial*>(reinterpret_cast<uint8_t*>(scratch) + kLookupHeaderBytes);
  int nparts = 0;
  if (N > 0) {
    nparts = (int)scan_blocks(N);
    hipLaunchKernelGGL(lookup_scan_kernel, dim3((unsigned)nparts), dim3(kWaves * 64), 0, s, cache_emb, query, N, d, partial,
                       qnorm2);
    CHORUS_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(lookup_final_kernel, dim3(1), dim3(256), 0, s, partial, nparts, qnorm2, N, tau, out);
  CHORUS_LAUNCH_CHECK();
  return CHORUS_OK;
}

// Scratch of the entry point that allocates nothing: the header and the largest number of partials a scan leaves
// (the scan caps its grid, so this serves every N). One copy per GPU, resident until the process ends.
constexpr size_t kStaticScratchBytes = kLookupHeaderBytes + (size_t)kMaxScanBlocks * sizeof(LookupPartial);
static __device__ __align__(256) uint8_t scratch[kStaticScratchBytes];

// Device address of `scratch` on each GPU. In host code the array's name is only a handle for
// hipGetSymbolAddress; the address it returns for the current device is what kernels are given.
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

int32_t static_scratch(void** ptr) {
  int dev = -1;
  CHORUS_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return CHORUS_E_SHAPE;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {  // first call on this device (racing first calls resolve the same address)
    CHORUS_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return CHORUS_E_HIP;
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  return CHORUS_OK;
}

int32_t check_lookup_args(const float* cache_emb, int64_t N, int32_t d, const float* query, const chorus_lookup_result* out) {
  if (N < 0 || d <= 0 || !out || !query) return CHORUS_E_ARG;
  if (N > 0 && !cache_emb) return CHORUS_E_ARG;
  if ((d & 3) != 0) return CHORUS_E_SHAPE;
  if (N > 0x7fffffffLL - 1) return CHORUS_E_SHAPE;  // the result index is an int32
  if (!aligned16(cache_emb) || !aligned16(query)) return CHORUS_E_ARG;
  return CHORUS_OK;
}

}  // namespace
}  // namespace chorus

using namespace chorus;

extern "C" {

int32_t chorus_version(void) { return 100; }
int32_t chorus_last_hip_error(void) { return g_last_hip_error; }

size_t chorus_cache_lookup_workspace_bytes(int64_t N) { return lookup_scratch_bytes(N > 0 ? (long)N : 0); }

int32_t chorus_cache_lookup(const float* cache_emb, int64_t N, int32_t d, const float* query, float tau,
                            chorus_lookup_result* out, void* ws, size_t ws_bytes, void* stream) {
  CHK_STATUS(check_lookup_args(cache_emb, N, d, query, out));
  if (!ws || ws_bytes < chorus_cache_lookup_workspace_bytes(N)) return CHORUS_E_WORKSPACE;
  if (!aligned16(ws)) return CHORUS_E_ARG;
  return launch_lookup(cache_emb, (long)N, d, query, tau, out, ws, (hipStream_t)stream);
}

int32_t chorus_cache_lookup_static(const float* cache_emb, int64_t N, int32_t d, const float* query, float tau,
                                   chorus_lookup_result* out, void* stream) {
  CHK_STATUS(check_lookup_args(cache_emb, N, d, query, out));
  if (lookup_scratch_bytes(N > 0 ? (long)N : 0) > kStaticScratchBytes) return CHORUS_E_SHAPE;
  void* ptr = nullptr;
  CHK_STATUS(static_scratch(&ptr));
  // nothing in the scratch has to start at zero: the scan writes the query norm and every partial the final
  // kernel reads (it reads as many as this call's scan has workgroups), so what an earlier call left is never seen
  return launch_lookup(cache_emb, (long)N, d, query, tau, out, ptr, (hipStream_t)stream);
}

}  // extern "C"
