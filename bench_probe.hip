// Benchmark helper, built into a small library of its own (libbench_probe.so) that only bench.py
// loads; the layer library does not contain it.  A register-only loop of matrix instructions: no
// memory traffic inside the loop, so the rate it reaches is what the matrix pipes deliver at the
// clock the chip sustains under that load -- the practical ceiling the GEMM kernels are compared
// with beside the published peak.
//
//   int bench_mfma_probe(int f64, int32_t workgroups, int32_t iters, uint64_t* out, int32_t* timer_khz,
//                        void* hip_stream)
// `workgroups` workgroups of four waves each run `iters` rounds of four independent matrix
// instructions (32x32x2 fp32, or 16x16x4 fp64 when f64 != 0) on registers only.  Wave v of workgroup
// b writes two counts to out[2*(4*b + v)] and out[2*(4*b + v) + 1]: the core-clock ticks and the
// ticks of the device's constant-rate timer that its loop took.  `out` is device memory of
// 8*workgroups uint64, caller-owned; `timer_khz` (host pointer, may be NULL) receives the rate of
// that timer.  FLOPs of one launch = workgroups * 4 * iters * 4 * (4096 fp32 | 2048 fp64).
// Enqueued on hip_stream without synchronising.  Returns 0, -1 for a null `out`, workgroups outside
// [1, 65536] or iters outside [1, 2^20], or a positive hipError_t.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, uint64_t* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  // operands with varied mantissas; the sums stay far from overflow for any allowed iteration count
  const float a0 = 1.0f + (float)lane * 0.0009765625f, a1 = 0.5f + (float)lane * 0.001953125f;
  const float b0 = 1.52587890625e-05f * (float)(lane + 1), b1 = 3.0517578125e-05f * (float)(64 - lane);
  f32x16 c0 = {}, c1 = {}, c2 = {}, c3 = {};
  const uint64_t t0 = clock64(), r0 = wall_clock64();
  for (int i = 0; i < iters; ++i) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, c3, 0, 0, 0);
  }
  asm volatile("" ::"v"(c0), "v"(c1), "v"(c2), "v"(c3));  // the products are needed: keep the loop
  const uint64_t t1 = clock64(), r1 = wall_clock64();
  if (lane == 0) {
    const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    out[2 * wave] = t1 - t0;
    out[2 * wave + 1] = r1 - r0;
  }
}

typedef double f64x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void mfma_probe64_kernel(int iters, uint64_t* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const double a0 = 1.0 + (double)lane * 0.0009765625, a1 = 0.5 + (double)lane * 0.001953125;
  const double b0 = 1.52587890625e-05 * (double)(lane + 1), b1 = 3.0517578125e-05 * (double)(64 - lane);
  f64x4 c0 = {}, c1 = {}, c2 = {}, c3 = {};
  const uint64_t t0 = clock64(), r0 = wall_clock64();
  for (int i = 0; i < iters; ++i) {
    c0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, c3, 0, 0, 0);
  }
  asm volatile("" ::"v"(c0), "v"(c1), "v"(c2), "v"(c3));
  const uint64_t t1 = clock64(), r1 = wall_clock64();
  if (lane == 0) {
    const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    out[2 * wave] = t1 - t0;
    out[2 * wave + 1] = r1 - r0;
  }
}

}  // namespace

extern "C" int bench_mfma_probe(int f64, int32_t workgroups, int32_t iters, uint64_t* out, int32_t* timer_khz,
                                void* hip_stream) {
  if (!out || workgroups < 1 || workgroups > 65536 || iters < 1 || iters > (1 << 20)) return -1;
  if (timer_khz) {
    int dev = 0, khz = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev);
    if (e != hipSuccess) return (int)e;
    *timer_khz = khz;
  }
  if (f64)
    hipLaunchKernelGGL(mfma_probe64_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream, iters, out);
  else
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream, iters, out);
  return (int)hipGetLastError();
}
