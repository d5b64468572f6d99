// Small HBM-bound helpers of the InnerProduct layer (paper Table 1, Appendix A/B): the ReLU's
// gradient mask and the column sums of the bias gradient.  The layer's three contractions run on
// the correlation and filter-gradient kernels with the operand roles exchanged.
#include <hip/hip_runtime.h>

#include "internal.h"

namespace mi355conv {

namespace {

// dz = y > 0 ? dy : 0 (a plain copy when y is null), four elements per thread where the count allows.
__global__ __launch_bounds__(256) void relu_bwd_kernel(const ReluBwdArgs a) {
  const int i4 = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (a.y == nullptr) {
    for (int i = i4; i < i4 + 4 && i < a.count; ++i) a.dz[i] = a.dy[i];
  } else if (i4 + 3 < a.count) {
    const float4 y = *reinterpret_cast<const float4*>(a.y + i4);
    float4 g = *reinterpret_cast<const float4*>(a.dy + i4);
    g.x = y.x > 0.f ? g.x : 0.f;
    g.y = y.y > 0.f ? g.y : 0.f;
    g.z = y.z > 0.f ? g.z : 0.f;
    g.w = y.w > 0.f ? g.w : 0.f;
    *reinterpret_cast<float4*>(a.dz + i4) = g;
  } else {
    for (int i = i4; i < a.count; ++i) a.dz[i] = a.y[i] > 0.f ? a.dy[i] : 0.f;
  }
}

// part[s][c] = sum of src[r][c] over the rows of split s.  One thread per column (coalesced along
// the row), four independent accumulators; the splits are added in order by the reduce kernel.
__global__ __launch_bounds__(256) void colsum_kernel(const ColSumArgs a) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  const int s = blockIdx.y;
  if (c >= a.cols) return;
  const int r0 = s * a.rows_per_split;
  int r1 = r0 + a.rows_per_split;
  if (r1 > a.rows) r1 = a.rows;
  const float* src = a.src + c;
  float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
  int r = r0;
  for (; r + 3 < r1; r += 4) {
    acc0 += src[(size_t)r * a.cols];
    acc1 += src[(size_t)(r + 1) * a.cols];
    acc2 += src[(size_t)(r + 2) * a.cols];
    acc3 += src[(size_t)(r + 3) * a.cols];
  }
  for (; r < r1; ++r) acc0 += src[(size_t)r * a.cols];
  a.part[(size_t)s * a.cols + c] = (acc0 + acc1) + (acc2 + acc3);
}

// Small matrices: dst[c] = beta*dst[c] + sum over all rows of src[r][c] in one launch.  A block
// owns 64 columns; its four waves take every fourth row (four loads in flight per lane) and the
// four partial sums are added in wave order.
__global__ __launch_bounds__(256) void colsum_direct_kernel(const ColSumArgs a) {
  __shared__ float part[4][64];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
  if (c < a.cols) {
    const float* src = a.src + c;
    int r = wv;
    for (; r + 12 < a.rows; r += 16) {
      acc0 += src[(size_t)r * a.cols];
      acc1 += src[(size_t)(r + 4) * a.cols];
      acc2 += src[(size_t)(r + 8) * a.cols];
      acc3 += src[(size_t)(r + 12) * a.cols];
    }
    for (; r < a.rows; r += 4) acc0 += src[(size_t)r * a.cols];
  }
  part[wv][lane] = (acc0 + acc1) + (acc2 + acc3);
  __syncthreads();
  if (wv == 0 && c < a.cols) {
    const float s = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
    a.dst[c] = a.beta != 0.f ? a.beta * a.dst[c] + s : s;
  }
}

}  // namespace

int launch_relu_bwd(const ReluBwdArgs& a, void* stream) {
  const int blocks = (a.count + 1023) / 1024;
  if (blocks == 0) return 0;
  hipLaunchKernelGGL(relu_bwd_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

int launch_colsum(const ColSumArgs& a, void* stream) {
  if (a.dst) {
    hipLaunchKernelGGL(colsum_direct_kernel, dim3((a.cols + 63) / 64), dim3(256), 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
  }
  hipLaunchKernelGGL(colsum_kernel, dim3((a.cols + 255) / 256, a.S), dim3(256), 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

}  // namespace mi355conv
