// Device-side helpers for the gfx950 kernels: fp32 MFMA wrappers, magic division, XCD-aware
// block renumbering.
#pragma once

#include <hip/hip_runtime.h>

#include <mutex>

#include "internal.h"

namespace mi355conv {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t mdiv(uint32_t x, Magic m) { return (__umulhi(x, m.mul) + x) >> m.shift; }

// fp32 matrix instructions of CDNA: one wave computes D += A*B with
//   MT = 32: 32x32 tile, 2 k-values per instruction (lane l feeds A[l%32][l/32], B[l/32][l%32]),
//            16 accumulators per lane: register r holds D[8*(r/4) + 4*(l/32) + r%4][l%32]
//   MT = 16: 16x16 tile, 4 k-values per instruction (lane l feeds A[l%16][l/16], B[l/16][l%16]),
//            4 accumulators per lane: register r holds D[4*(l/16) + r][l%16]
template <int MT>
struct Mfma;

template <>
struct Mfma<32> {
  using Acc = f32x16;
  static constexpr int KS = 2;   // reduction depth of one instruction
  static constexpr int NR = 16;  // accumulator registers per lane
  static __device__ __forceinline__ void run(float a, float b, Acc& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ int row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }
};

template <>
struct Mfma<16> {
  using Acc = f32x4;
  static constexpr int KS = 4;
  static constexpr int NR = 4;
  static __device__ __forceinline__ void run(float a, float b, Acc& c) {
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ int row(int r, int lane) { return 4 * (lane >> 4) + r; }
};

// Consecutive workgroup ids are handed to the 8 XCDs in turn, and each XCD has its own L2.
// Renumber so that each XCD works on one contiguous run of logical tiles (neighbouring tiles
// share gathered input rows and the packed weights).
__device__ __forceinline__ uint32_t xcd_contiguous_block_id() {
  const uint32_t nb = gridDim.x, bid = blockIdx.x;
  const uint32_t q = nb >> 3, r = nb & 7u, x = bid & 7u, idx = bid >> 3;
  return x * q + (x < r ? x : r) + idx;
}

// Load with an unsigned 32-bit byte offset from a uniform base (one address register per lane).
__device__ __forceinline__ float ld_f32(const float* base, uint32_t byte_off) {
  return *reinterpret_cast<const float*>(reinterpret_cast<const char*>(base) + byte_off);
}

// One-time opt-in of a kernel to more than 64 KB of dynamic LDS.  The first launch of a kernel
// instance performs it (a host-side attribute call, not an enqueue -- so that first launch must not
// happen inside a stream capture); std::call_once makes it safe for threads that share a descriptor.
struct LdsOptIn {
  std::once_flag once;
  int err = 0;
};

template <typename Kernel>
inline int lds_opt_in(LdsOptIn& state, Kernel kernel, int bytes) {
  std::call_once(state.once, [&] {
    state.err = (int)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  });
  return state.err;
}

}  // namespace mi355conv
