// Small device helpers shared by the HIP kernels (gfx950, 64-lane wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <atomic>
#include <cstdint>
#include <mutex>

#include "kernels.hpp"

namespace ls {

// kernel<<<grid, block, smem, st>>>(args...), or the same launch with the runtime's per-kernel
// start/stop events when the stage runtime has armed launch_timing().
template <typename... KArgs, typename... Args>
inline void launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, unsigned smem, hipStream_t st, Args... args) {
  LaunchTiming& t = launch_timing();
  if (t.start) {
    hipExtLaunchKernelGGL(kernel, grid, block, smem, st, t.start, t.stop, 0, static_cast<KArgs>(args)...);
    t.start = t.stop = nullptr;
    t.used = true;
  } else {
    hipLaunchKernelGGL(kernel, grid, block, smem, st, static_cast<KArgs>(args)...);
  }
}

// Raise a kernel's dynamic-LDS limit, once per device (`done` holds one bit per device ordinal;
// the attribute belongs to each device's copy of the kernel).  Safe from several threads: a
// race only sets the same attribute twice.
inline void allow_dynamic_lds(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  (void)hipGetDevice(&dev);
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return;
  (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  done.fetch_or(bit, std::memory_order_release);
}

// The same for a kernel whose LDS need varies with the shape: `allowed[device]` is the limit set
// so far, raised (under a lock, so that a smaller request cannot overwrite a larger one) when a
// launch needs more.
inline void allow_dynamic_lds_up_to(const void* kernel, int bytes, std::atomic<int> (&allowed)[64]) {
  static std::mutex m;
  int dev = 0;
  (void)hipGetDevice(&dev);
  std::atomic<int>& a = allowed[dev & 63];
  if (bytes <= a.load(std::memory_order_acquire)) return;
  std::lock_guard<std::mutex> lock(m);
  if (bytes <= a.load(std::memory_order_relaxed)) return;
  (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  a.store(bytes, std::memory_order_release);
}

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // a raw 16-byte load
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float to_f(float v) { return v; }
__device__ __forceinline__ float to_f(bf16 v) { return (float)v; }
// float -> storage type; the bf16 conversion rounds to nearest, ties to even.
template <class T> __device__ __forceinline__ T from_f(float f);
template <> __device__ __forceinline__ float from_f<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16 from_f<bf16>(float f) { return (bf16)f; }

// Sum over the 64 lanes of a wavefront; every lane gets the total (fixed butterfly order).
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}

// Sum over each aligned group of 16 lanes, every lane of the group gets the total.  Four
// register-to-register DPP exchanges (lane^1, lane^2, mirrored half row, mirrored row) in a
// fixed order -- no trip through the LDS crossbar as with a general shuffle.
__device__ __forceinline__ float row16_sum(float v) {
#define LS_DPP_ADD(ctrl) \
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, 0xF, 0xF, true))
  LS_DPP_ADD(0xB1);   // quad_perm [1,0,3,2]
  LS_DPP_ADD(0x4E);   // quad_perm [2,3,0,1]
  LS_DPP_ADD(0x141);  // row_half_mirror: the other quad of the half row
  LS_DPP_ADD(0x140);  // row_mirror: the other half row
#undef LS_DPP_ADD
  return v;
}

// silu(z) = z / (1 + exp(-z)), the quotient as a product with the hardware reciprocal (1 ulp):
// a correctly rounded fp32 division is ten instructions, and every result is rounded to bf16
__device__ __forceinline__ float silu_f(float z) { return z * __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }

}  // namespace ls
