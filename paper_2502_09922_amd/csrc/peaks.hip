// Measurement aids (not part of the stage's path): what this GPU sustains for the two
// resources the path is bound by, measured with the same instructions the kernels use.
//   * a streaming read of a device buffer with 16-byte non-temporal loads, as the decode
//     kernels read weights and cached keys / values;
//   * a register-only loop of v_mfma_f32_16x16x32_bf16 on every SIMD, the instruction the
//     prompt GEMM issues, with no operand traffic at all and with operands that differ from
//     lane to lane (dense MFMA work is power-bound on this chip and all-zero or constant
//     operands let it hold a clock that real data does not: 2.4 GHz against about 2.15).
// bench.py reports its fractions against the published peaks and against these.
#include "../../include/ls_stage.h"
#include "kernels.hpp"
#include "device_util.hpp"

#include <cstdio>
#include <cstdlib>

namespace {

constexpr int READ_WGS = 256 * 8;  // workgroups of the read probe: eight per CU
constexpr int MFMA_WGS = 256 * 2;  // workgroups of the MFMA probe: two per CU, one wave per SIMD each

__global__ void __launch_bounds__(256) k_probe_read(const ls::u32x4* __restrict__ p, size_t n16, unsigned* sink) {
  ls::u32x4 a = {0u, 0u, 0u, 0u};
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  // four independent loads in flight per lane
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const ls::u32x4 v0 = __builtin_nontemporal_load(p + i);
    const ls::u32x4 v1 = __builtin_nontemporal_load(p + i + stride);
    const ls::u32x4 v2 = __builtin_nontemporal_load(p + i + 2 * stride);
    const ls::u32x4 v3 = __builtin_nontemporal_load(p + i + 3 * stride);
    a ^= v0 ^ v1 ^ v2 ^ v3;
  }
  for (; i < n16; i += stride) a ^= __builtin_nontemporal_load(p + i);
  // never true for the all-ones pattern below unless the buffer says so; keeps the loads alive
  if (sink && (a[0] & a[1] & a[2] & a[3]) == 0xffffffffu) sink[0] = a[0];
}

__global__ void __launch_bounds__(256) k_probe_mfma(int iters, float seed, float* sink) {
  ls::f32x4 acc[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) acc[j] = ls::f32x4{0.f, 0.f, 0.f, 0.f};
  ls::bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (ls::bf16)(seed + (float)((threadIdx.x * 7 + e * 13) % 31) * 0.03f - 0.4f);
    b[e] = (ls::bf16)(seed + (float)((threadIdx.x * 5 + e * 11) % 29) * 0.02f - 0.3f);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 16; ++j) s += acc[j][0] + acc[j][3];
  if (sink && s == 12345.678f) sink[0] = s;  // keeps the accumulators alive
}

// best of `reps` timings of `launch` on `st`, in milliseconds; negative on a HIP error
template <class F>
double best_ms(int reps, hipStream_t st, F launch) {
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess) return -1.0;
  if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return -1.0; }
  double best = -1.0;
  bool ok = true;
  for (int r = 0; r <= reps && ok; ++r) {  // rep 0 warms up
    ok = hipEventRecord(a, st) == hipSuccess;
    launch();
    ok = ok && hipEventRecord(b, st) == hipSuccess && hipEventSynchronize(b) == hipSuccess;
    float ms = 0.f;
    ok = ok && hipEventElapsedTime(&ms, a, b) == hipSuccess && hipGetLastError() == hipSuccess;
    if (ok && r > 0 && (best < 0 || ms < best)) best = ms;
  }
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  return ok ? best : -1.0;
}

}  // namespace

extern "C" {

double ls_probe_read_gbps(const void* buf, size_t bytes, int reps, void* sink, void* hip_stream) {
  if (!buf || bytes < 16 || reps < 1 || ((uintptr_t)buf & 15)) {
    ls::set_last_error("ls_probe_read_gbps: bad arguments");
    return -1.0;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t n16 = bytes / 16;
  // the best of a few grid sizes (8 to 256 workgroups per CU): the fastest differs with the size of the buffer
  double ms = -1.0;
  for (int wgs = READ_WGS; wgs <= READ_WGS * 32; wgs *= 2) {
    const double t = best_ms(reps, st, [&] {
      k_probe_read<<<wgs, 256, 0, st>>>((const ls::u32x4*)buf, n16, (unsigned*)sink);
    });
    if (t <= 0) {
      ls::set_last_error("ls_probe_read_gbps: HIP error");
      return -1.0;
    }
    if (ms < 0 || t < ms) ms = t;
  }
  return (double)(n16 * 16) / (ms * 1e-3) / 1e9;
}

double ls_probe_mfma_tflops(int iters, int reps, void* sink, void* hip_stream) {
  if (iters < 1 || reps < 1) {
    ls::set_last_error("ls_probe_mfma_tflops: bad arguments");
    return -1.0;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  const double ms = best_ms(reps, st, [&] { k_probe_mfma<<<MFMA_WGS, 256, 0, st>>>(iters, 0.f, (float*)sink); });
  if (ms <= 0) {
    ls::set_last_error("ls_probe_mfma_tflops: HIP error");
    return -1.0;
  }
  const double flops = (double)MFMA_WGS * 4 /*waves*/ * iters * 16 * (2.0 * 16 * 16 * 32);
  return flops / (ms * 1e-3) / 1e12;
}

}  // extern "C"
