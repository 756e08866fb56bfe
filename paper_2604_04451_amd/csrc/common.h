// Shared host/device helpers of the Chorus HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "chorus.h"

namespace chorus {

// last HIP error seen by this library on this thread
extern thread_local int32_t g_last_hip_error;

inline int32_t hip_fail(hipError_t e) {
  g_last_hip_error = (int32_t)e;
  return CHORUS_E_HIP;
}

#define CHORUS_HIP(expr)                                   \
  do {                                                     \
    hipError_t e__ = (expr);                               \
    if (e__ != hipSuccess) return ::chorus::hip_fail(e__); \
  } while (0)

#define CHORUS_LAUNCH_CHECK() CHORUS_HIP(hipGetLastError())

#define CHK_STATUS(call)                    \
  do {                                      \
    int32_t st__ = (call);                  \
    if (st__ != CHORUS_OK) return st__;     \
  } while (0)

// Raises a kernel's dynamic-LDS limit once per device. The limit is a property of the (kernel, device) pair, so the
// record is a bit per device ordinal; setting it twice from racing threads is harmless (same value), and a device
// ordinal beyond the mask is simply set on every call.
struct DynLdsOnce {
  std::atomic<uint64_t> done{0};
  int32_t ensure(const void* kernel, int bytes) {
    int dev = 0;
    CHORUS_HIP(hipGetDevice(&dev));
    const uint64_t bit = (dev >= 0 && dev < 64) ? (1ull << dev) : 0ull;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return CHORUS_OK;
    CHORUS_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    if (bit) done.fetch_or(bit, std::memory_order_release);
    return CHORUS_OK;
  }
};

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Base address of a workspace that is being carved into regions. The base is null when only the total size is
// wanted, and offsetting a null pointer is undefined, so the addresses are formed in integer arithmetic.
struct BytePtr {
  uintptr_t addr;
  explicit BytePtr(void* p) : addr(reinterpret_cast<uintptr_t>(p)) {}
  uint8_t* operator+(size_t off) const { return reinterpret_cast<uint8_t*>(addr + off); }
};

typedef __bf16 bf16_t;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
// plain 16-byte register vector (HIP's uint4 is a struct and keeps arrays of it out of registers)
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

// streaming (non-temporal) 16-byte accesses for data touched once
__device__ __forceinline__ float4 ld_stream_f4(const float4* p) {
  f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
  return make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void st_stream_f4(float4* p, float4 a) {
  f32x4 v = {a.x, a.y, a.z, a.w};
  __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(p));
}

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round to nearest even; the compiler emits the hardware convert on gfx950
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  bf16_t h = (bf16_t)f;
  return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// value of the lane 32 away (lanes l and l ^ 32 exchange): one register-file swap instruction instead of a trip
// through the LDS crossbar
__device__ __forceinline__ float swap_halves(float v) {
  const uint32_t b = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane32_swap(b, b, false, false);  // r[0] = (lo, lo), r[1] = (hi, hi)
  return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

// value of the lane 16 away (lanes l and l ^ 16 exchange), likewise one register-file swap instruction
__device__ __forceinline__ float swap_rows16(float v) {
  const uint32_t b = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane16_swap(b, b, false, false);  // r[0] = rows (0, 0, 2, 2), r[1] = rows (1, 1, 3, 3)
  return __uint_as_float((threadIdx.x & 16) ? r[0] : r[1]);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Workgroup barrier that orders LDS traffic only: waits for this wave's LDS operations
// (lgkmcnt) but leaves global loads in flight, unlike __syncthreads(), whose fences also
// drain vmcnt and would expose the latency of every prefetch. The fences keep the compiler
// from moving LDS accesses across the barrier.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Workgroup id -> logical tile id such that the workgroups that land on one XCD
// (hardware deals consecutive ids round-robin over the 8 XCDs) cover one
// contiguous range of logical ids and so share operands in that XCD's L2.
__device__ __forceinline__ int xcd_remap(int bid, int nblocks) {
  const int NX = 8;
  int xcd = bid % NX, local = bid / NX;
  int q = nblocks / NX, r = nblocks % NX;
  // XCD x owns q+1 ids if x < r else q ids
  int start = xcd * q + (xcd < r ? xcd : r);
  return start + local;
}

}  // namespace chorus
