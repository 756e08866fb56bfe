// Measured matrix-pipe ceiling of the part for benchmarks: a loop of nothing but
// v_mfma_f32_16x16x32_bf16 (two waves per SIMD, every CU; every result block accumulated by four MFMAs
// in a row), optionally with the two companions the self-attention kernel cannot avoid -- one 1 KB
// operand read from LDS per two MFMAs and one exp2 + maximum per two MFMAs (per logit). The sustained
// rate depends on the operand VALUES: the chip is power-managed, constant operands run at the nominal
// rate, random ones far below it. The roofline fraction of a kernel is quoted against the published
// peak; this number says how much of that peak the silicon sustains for a given instruction mix and data.
#include "chorus_ops.h"
#include "common.h"

namespace chorus {
namespace {

constexpr int kCeilThreads = 512;
constexpr int kCeilIters = 2000;  // x 64 MFMAs per wave per launch

__device__ inline float hash_normal(unsigned idx) {
  unsigned h = idx * 2654435761u + 0x9E3779B9u;
  h ^= h >> 15; h *= 0x2C1B3C6Du; h ^= h >> 12; h *= 0x297A2D39u; h ^= h >> 15;
  unsigned g = h * 0x85EBCA6Bu + 0xC2B2AE35u;
  g ^= g >> 13; g *= 0xC2B2AE35u; g ^= g >> 16;
  const float u1 = ((h >> 8) + 1.0f) * (1.0f / 16777217.0f);
  const float u2 = (g >> 8) * (1.0f / 16777216.0f);
  return sqrtf(-2.0f * __logf(u1)) * __cosf(6.2831853f * u2);
}

// MIX bit 0: the A operand of every pair of MFMAs comes from LDS; bit 1: exp2 + max per pair of MFMAs
template <int MIX>
__global__ __launch_bounds__(kCeilThreads) void mfma_ceiling_kernel(float* __restrict__ out, int normal_data, int iters) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[8 * kCeilThreads * 8];
  bf16x8 a[8], b[4];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i)
      a[j][i] = (bf16_t)(normal_data ? hash_normal((j * kCeilThreads + threadIdx.x) * 8 + i) : 1.0f);
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i)
      b[j][i] = (bf16_t)(normal_data ? hash_normal(((8 + j) * kCeilThreads + threadIdx.x) * 8 + i) : 1.0f);
#pragma unroll
  for (int j = 0; j < 8; ++j) *reinterpret_cast<bf16x8*>(lds + ((size_t)j * kCeilThreads + threadIdx.x) * 8) = a[j];
  __syncthreads();
  float e[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) e[i] = (float)a[i][0];
  float emax = 0.f;
  f32x4 c[4][4] = {};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < 4; ++t)  // 4 x 16 MFMAs = the flops of 32 MFMAs of the 32x32x16 shape
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        bf16x8 av[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          av[ks] = a[4 * h + ks];
          if (MIX & 1)
            av[ks] = *reinterpret_cast<const bf16x8*>(
                lds + ((size_t)(4 * h + ks) * kCeilThreads + ((threadIdx.x + 64 * t) & (kCeilThreads - 1))) * 8);
        }
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) {  // four MFMAs in a row into one result block
            c[t][2 * h + r] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[ks], b[(ks + r) & 3], c[t][2 * h + r], 0, 0, 0);
            if ((MIX & 2) && r == 0) {
              const float p = __builtin_amdgcn_exp2f(-e[4 * h + ks]);
              emax = fmaxf(emax, p);
              e[4 * h + ks] = p;
            }
          }
      }
    __builtin_amdgcn_sched_barrier(0);
  }
  float s = emax;
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) s += c[t][j][i];
  out[(size_t)blockIdx.x * kCeilThreads + threadIdx.x] = s;
}

template <int MIX>
void launch_ceiling(float* out, int grid, int normal_data, hipStream_t s) {
  hipLaunchKernelGGL(mfma_ceiling_kernel<MIX>, dim3(grid), dim3(kCeilThreads), 0, s, out, normal_data, kCeilIters);
}

}  // namespace
}  // namespace chorus

using namespace chorus;

extern "C" {

size_t chorus_mfma_ceiling_workspace_bytes(void) { return (size_t)1024 * kCeilThreads * sizeof(float); }

int32_t chorus_mfma_ceiling(int32_t normal_data, int32_t mix, int32_t launches, double* tflops, void* ws, size_t ws_bytes,
                            void* stream) {
  if (!tflops || mix < 0 || mix > 3 || launches < 1 || launches > 1000) return CHORUS_E_ARG;
  if (!ws || ws_bytes < chorus_mfma_ceiling_workspace_bytes()) return CHORUS_E_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  int dev = 0, cus = 0;
  CHORUS_HIP(hipGetDevice(&dev));
  CHORUS_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  if (cus < 1 || cus > 1024) return CHORUS_E_SHAPE;
  float* out = (float*)ws;
  auto go = [&](int n) {
    for (int r = 0; r < n; ++r) switch (mix) {
        case 0: launch_ceiling<0>(out, cus, normal_data != 0, s); break;
        case 1: launch_ceiling<1>(out, cus, normal_data != 0, s); break;
        case 2: launch_ceiling<2>(out, cus, normal_data != 0, s); break;
        default: launch_ceiling<3>(out, cus, normal_data != 0, s); break;
      }
  };
  hipEvent_t e0, e1;
  CHORUS_HIP(hipEventCreate(&e0));
  CHORUS_HIP(hipEventCreate(&e1));
  go(2 * launches);  // the clock settles over tens of milliseconds: warm up for twice the timed span
  CHORUS_HIP(hipEventRecord(e0, s));
  go(launches);
  CHORUS_HIP(hipEventRecord(e1, s));
  CHORUS_LAUNCH_CHECK();
  CHORUS_HIP(hipEventSynchronize(e1));
  float ms = 0.f;
  CHORUS_HIP(hipEventElapsedTime(&ms, e0, e1));
  hipEventDestroy(e0);
  hipEventDestroy(e1);
  const double flops = (double)cus * (kCeilThreads / 64) * kCeilIters * 64.0 * (2.0 * 16 * 16 * 32) * launches;
  *tflops = ms > 0.f ? flops / ((double)ms * 1e9) : 0.0;
  return CHORUS_OK;
}

}  // extern "C"
