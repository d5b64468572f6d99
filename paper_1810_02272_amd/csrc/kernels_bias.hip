// Bias gradient of the Caffe-semantics convolution layer (paper Table 1):
//   db[k] = beta*db[k] + sum over n, oh, ow of dy[n,k,oh,ow]
// One read of dy, so HBM-bound.  Stage 1: grid (K, S) -- each workgroup sums channel k over a
// slice of the batch with a wave-level DPP reduction and writes part[s][k]; stage 2 (the shared
// reduce kernel) adds the S partials in order and applies beta.
#include <hip/hip_runtime.h>

#include "device_utils.h"
#include "internal.h"

namespace mi355conv {

namespace {

// Sum over the 64 lanes of a wave; every lane of row 0 returns the total.
__device__ __forceinline__ float wave_sum(float v) {
  // within quads: xor 1, xor 2; within rows of 16: half mirror, mirror
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, false));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, false));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, false));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, false));
  // the four row sums
  const int iv = __builtin_bit_cast(int, v);
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 0)) +
         __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 16)) +
         __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 32)) +
         __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 48));
}

__global__ __launch_bounds__(256) void bias_grad_kernel(const BiasGradArgs a) {
  __shared__ float wsum[4];
  const int k = blockIdx.x, s = blockIdx.y;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int n0 = s * a.n_per_split;
  int n1 = n0 + a.n_per_split;
  if (n1 > a.N) n1 = a.N;
  // Each wave walks whole images (one contiguous run of P floats per image and channel), the four
  // waves of the block taking every fourth image; four independent accumulators per lane keep
  // several loads in flight.
  // A plane starts on an arbitrary 4-byte boundary: up to three leading elements, then 16-byte
  // loads, then up to three trailing elements.
  float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
  for (int n = n0 + wv; n < n1; n += 4) {
    const float* src = a.dy + ((size_t)n * a.K + k) * a.P;
    if (a.P < 512 && (a.P & 3) != 0) {  // small planes that start off 16-byte boundaries: head and tail cost more than they save
      for (int p = lane; p < a.P; p += 64) acc0 += src[p];
      continue;
    }
    int head = (int)((0u - (uint32_t)(reinterpret_cast<uintptr_t>(src) >> 2)) & 3u);
    if (lane < head) acc0 += src[lane];
    const float4* v = reinterpret_cast<const float4*>(src + head);
    const int nvec = (a.P - head) >> 2;
    int i = lane;
    for (; i + 192 < nvec; i += 256) {
      const float4 x0 = v[i], x1 = v[i + 64], x2 = v[i + 128], x3 = v[i + 192];
      acc0 += (x0.x + x0.y) + (x0.z + x0.w);
      acc1 += (x1.x + x1.y) + (x1.z + x1.w);
      acc2 += (x2.x + x2.y) + (x2.z + x2.w);
      acc3 += (x3.x + x3.y) + (x3.z + x3.w);
    }
    for (; i < nvec; i += 64) {
      const float4 x0 = v[i];
      acc1 += (x0.x + x0.y) + (x0.z + x0.w);
    }
    const int tail = head + 4 * nvec + lane;
    if (tail < a.P) acc2 += src[tail];
  }
  const float w = wave_sum((acc0 + acc1) + (acc2 + acc3));
  if (lane == 0) wsum[wv] = w;
  __syncthreads();
  if (threadIdx.x == 0) {
    const float total = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
    if (a.db)
      a.db[k] = a.beta != 0.f ? a.beta * a.db[k] + total : total;
    else
      a.part[(size_t)s * a.K + k] = total;
  }
}

// Zero fill, 16 bytes per thread (the tail word by word).
__global__ __launch_bounds__(256) void fill_zero_kernel(float* __restrict__ dst, size_t words) {
  const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i + 3 < words) {
    *reinterpret_cast<float4*>(dst + i) = make_float4(0.f, 0.f, 0.f, 0.f);
  } else {
    for (size_t j = i; j < words; ++j) dst[j] = 0.f;
  }
}

}  // namespace

int launch_fill_zero(void* dst, size_t bytes, void* stream) {
  const size_t words = bytes / 4;
  if (words == 0) return 0;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((words + 1023) / 1024)), dim3(256), 0, (hipStream_t)stream,
                     static_cast<float*>(dst), words);
  return (int)hipGetLastError();
}

int launch_bias_grad(const BiasGradArgs& a, void* stream) {
  hipLaunchKernelGGL(bias_grad_kernel, dim3(a.K, a.S), dim3(256), 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

}  // namespace mi355conv
