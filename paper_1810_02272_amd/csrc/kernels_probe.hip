// Measurement helper (not on the layer path): a register-only loop of fp32 matrix instructions.
// No memory traffic inside the loop, so the rate it reaches is what the matrix pipes deliver at
// the clock the chip sustains under that load -- the practical ceiling the GEMM kernels are
// compared with beside the published peak.
#include <hip/hip_runtime.h>

#include "device_utils.h"
#include "internal.h"
#include "mi355conv.h"

namespace mi355conv {

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

int run_probe(bool f64, int32_t workgroups, int32_t iters, uint64_t* out, int32_t* timer_khz, void* hip_stream) {
  if (!out || workgroups < 1 || workgroups > 65536 || iters < 1 || iters > (1 << 20)) return CONV_EINVAL;
  if (timer_khz) {
    int dev = 0, khz = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev);
    if (e != hipSuccess) return record_hip_error((int)e);
    *timer_khz = khz;
  }
  if (f64)
    hipLaunchKernelGGL(mfma_probe64_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream, iters, out);
  else
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream, iters, out);
  const int e = (int)hipGetLastError();
  return e ? record_hip_error(e) : CONV_OK;
}

}  // namespace

}  // namespace mi355conv

extern "C" int conv_mfma_probe(int32_t workgroups, int32_t iters, uint64_t* out, int32_t* timer_khz, void* hip_stream) {
  return mi355conv::run_probe(false, workgroups, iters, out, timer_khz, hip_stream);
}

extern "C" int conv_mfma_probe_f64(int32_t workgroups, int32_t iters, uint64_t* out, int32_t* timer_khz,
                                   void* hip_stream) {
  return mi355conv::run_probe(true, workgroups, iters, out, timer_khz, hip_stream);
}
