// Policy-gradient loss arithmetic of the paper's reinforcement-learning trainer (Appendix A:
// Sigmoid model, Appendix B: Softmax model): action sampling, discounted rewards (a reverse
// recurrence per episode), Dlogps and the modulated Bottom.diff.  All of it is element-wise or a
// short scan: one read and one write per value, HBM-bound.
#include <hip/hip_runtime.h>
#include <math.h>

#include "device_utils.h"
#include "internal.h"
#include "mi355pg.h"

namespace mi355conv {

namespace {

// ---- step 3: action = (random < Aprob) ? 0 : 1 ----
__global__ __launch_bounds__(256) void pg_sample_kernel(const float* __restrict__ aprob,
                                                        const float* __restrict__ random, int32_t* __restrict__ action,
                                                        int steps) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t < steps) action[t] = random[t] < aprob[t] ? 0 : 1;
}

// ---- step 9: R[t] = reward[t] + gamma * R[t+1] inside each episode ----
// One wave per episode, walking it from its end in chunks of 64 steps (lane 63 = the chunk's last
// step).  Inside a chunk the recurrence is a weighted suffix sum, done in six shuffle rounds with
// the weights gamma^1, ^2, ^4 ... ^32; the value carried in from the later chunk enters as
// gamma * carry added to the last lane's reward before the rounds.  Four chunks are loaded at a
// time so that a long episode does not pay one memory latency per 64 steps.
constexpr int kChunksInFlight = 4;

__device__ __forceinline__ float suffix_scan(float v, int lane, const float (&gpow)[6]) {
#pragma unroll
  for (int i = 0; i < 6; ++i) {
    const int d = 1 << i;
    const float o = __shfl_down(v, d, 64);
    v += (lane + d < 64) ? gpow[i] * o : 0.f;
  }
  return v;
}

__global__ __launch_bounds__(256) void pg_discount_kernel(const float* __restrict__ reward,
                                                          const int32_t* __restrict__ offsets, int episodes,
                                                          int steps, float gamma, float* __restrict__ discounted) {
  const int lane = threadIdx.x & 63;
  const int e = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (e >= episodes) return;
  int b = offsets[e], end = offsets[e + 1];
  b = b < 0 ? 0 : (b > steps ? steps : b);
  end = end < b ? b : (end > steps ? steps : end);
  float gpow[6];
  gpow[0] = gamma;
#pragma unroll
  for (int i = 1; i < 6; ++i) gpow[i] = gpow[i - 1] * gpow[i - 1];
  float carry = 0.f;
  for (int hi = end; hi > b; hi -= 64 * kChunksInFlight) {
    float r[kChunksInFlight];
#pragma unroll
    for (int c = 0; c < kChunksInFlight; ++c) {
      const int t = hi - 64 * (c + 1) + lane;
      r[c] = (t >= b && t < end) ? reward[t] : 0.f;
    }
#pragma unroll
    for (int c = 0; c < kChunksInFlight; ++c) {
      const int t = hi - 64 * (c + 1) + lane;
      float v = r[c] + (lane == 63 ? gamma * carry : 0.f);
      v = suffix_scan(v, lane, gpow);
      if (t >= b && t < end) discounted[t] = v;
      carry = __shfl(v, 0, 64);
    }
  }
}

// ---- Sigmoid model, steps 8, 10, 11 ----
__global__ __launch_bounds__(256) void pg_sigmoid_kernel(const float* __restrict__ aprob,
                                                         const int32_t* __restrict__ action,
                                                         const float* __restrict__ discounted,
                                                         float* __restrict__ dlogps, float* __restrict__ bottom_diff,
                                                         int steps) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= steps) return;
  const float ap = aprob[t];
  const float d = action[t] == 0 ? 1.f - ap : 0.f - ap;
  if (dlogps) dlogps[t] = d;
  const float w = discounted ? discounted[t] : 1.f;
  bottom_diff[t] = -d * w;
}

// ---- Softmax model, steps 8, 10, 11 ----
// Up to 32 actions: a block takes 256 consecutive rows, stages them through LDS with coalesced
// loads (row stride padded to an odd number of words so that one row per lane is conflict-free),
// lets each thread do its own row, and streams the results back out the same way.
__global__ __launch_bounds__(256) void pg_softmax_rows_kernel(const float* __restrict__ logits,
                                                              const int32_t* __restrict__ action,
                                                              const float* __restrict__ discounted,
                                                              float* __restrict__ probs,
                                                              float* __restrict__ bottom_diff, int steps, int A,
                                                              Magic mA) {
  extern __shared__ float tile[];  // [256][A | 1], then a second copy for the gradient
  const int AP = A | 1;
  float* const ptile = tile;
  float* const dtile = tile + 256 * AP;
  const int row0 = blockIdx.x * 256;
  const int nrows = steps - row0 < 256 ? steps - row0 : 256;
  const int count = nrows * A;
  const size_t base = (size_t)row0 * A;
  for (int i = threadIdx.x; i < count; i += 256) {
    const int r = (int)mdiv((uint32_t)i, mA);
    ptile[r * AP + (i - r * A)] = logits[base + i];
  }
  __syncthreads();
  if ((int)threadIdx.x < nrows) {
    float* const l = ptile + threadIdx.x * AP;
    float* const g = dtile + threadIdx.x * AP;
    const int act = action[row0 + threadIdx.x];
    const float w = discounted ? discounted[row0 + threadIdx.x] : 1.f;
    float top = l[0];
    for (int a = 1; a < A; ++a) top = fmaxf(top, l[a]);
    float sum = 0.f;
    for (int a = 0; a < A; ++a) {
      const float ex = expf(l[a] - top);
      l[a] = ex;
      sum += ex;
    }
    const float inv = 1.f / sum;
    for (int a = 0; a < A; ++a) {
      const float p = l[a] * inv;
      l[a] = p;
      g[a] = (p - (a == act ? 1.f : 0.f)) * w;
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < count; i += 256) {
    const int r = (int)mdiv((uint32_t)i, mA);
    const int o = r * AP + (i - r * A);
    if (probs) probs[base + i] = ptile[o];
    bottom_diff[base + i] = dtile[o];
  }
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d, 64));
  return v;
}

__device__ __forceinline__ float wave_add(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// More than 32 actions: one wave per row, lanes along the row.
__global__ __launch_bounds__(256) void pg_softmax_wide_kernel(const float* __restrict__ logits,
                                                              const int32_t* __restrict__ action,
                                                              const float* __restrict__ discounted,
                                                              float* __restrict__ probs,
                                                              float* __restrict__ bottom_diff, int steps, int A) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= steps) return;
  const float* const l = logits + (size_t)t * A;
  float top = -INFINITY;
  for (int a = lane; a < A; a += 64) top = fmaxf(top, l[a]);
  top = wave_max(top);
  float sum = 0.f;
  for (int a = lane; a < A; a += 64) sum += expf(l[a] - top);
  sum = wave_add(sum);
  const float inv = 1.f / sum;
  const int act = action[t];
  const float w = discounted ? discounted[t] : 1.f;
  for (int a = lane; a < A; a += 64) {
    const float p = expf(l[a] - top) * inv;
    if (probs) probs[(size_t)t * A + a] = p;
    bottom_diff[(size_t)t * A + a] = (p - (a == act ? 1.f : 0.f)) * w;
  }
}

int done(void) {
  const int e = (int)hipGetLastError();
  return e ? record_hip_error(e) : CONV_OK;
}

}  // namespace

}  // namespace mi355conv

using namespace mi355conv;

extern "C" {

int pg_sigmoid_sample_action(const float* aprob, const float* random, int32_t* action, int32_t steps,
                             void* hip_stream) {
  if (steps < 0) return CONV_EINVAL;
  if (steps == 0) return CONV_OK;
  if (!aprob || !random || !action) return CONV_EINVAL;
  hipLaunchKernelGGL(pg_sample_kernel, dim3((steps + 255) / 256), dim3(256), 0, (hipStream_t)hip_stream, aprob, random,
                     action, steps);
  return done();
}

int pg_discount_rewards(const float* reward, const int32_t* episode_offsets, int32_t episodes, int32_t steps,
                        float gamma, float* discounted, void* hip_stream) {
  if (episodes < 0 || steps < 0) return CONV_EINVAL;
  if (episodes == 0 || steps == 0) return CONV_OK;
  if (!reward || !episode_offsets || !discounted) return CONV_EINVAL;
  hipLaunchKernelGGL(pg_discount_kernel, dim3((episodes + 3) / 4), dim3(256), 0, (hipStream_t)hip_stream, reward,
                     episode_offsets, episodes, steps, gamma, discounted);
  return done();
}

int pg_sigmoid_bottom_diff(const float* aprob, const int32_t* action, const float* discounted, float* dlogps,
                           float* bottom_diff, int32_t steps, void* hip_stream) {
  if (steps < 0) return CONV_EINVAL;
  if (steps == 0) return CONV_OK;
  if (!aprob || !action || !bottom_diff) return CONV_EINVAL;
  hipLaunchKernelGGL(pg_sigmoid_kernel, dim3((steps + 255) / 256), dim3(256), 0, (hipStream_t)hip_stream, aprob,
                     action, discounted, dlogps, bottom_diff, steps);
  return done();
}

int pg_softmax_bottom_diff(const float* logits, const int32_t* action, const float* discounted, float* probs,
                           float* bottom_diff, int32_t steps, int32_t actions, void* hip_stream) {
  if (steps < 0 || actions < 1) return CONV_EINVAL;
  if ((int64_t)steps * actions >= ((int64_t)1 << 31)) return CONV_ESHAPE;
  if (steps == 0) return CONV_OK;
  if (!logits || !action || !bottom_diff) return CONV_EINVAL;
  if (actions <= 32) {
    const size_t lds = (size_t)2 * 256 * (actions | 1) * sizeof(float);  // at most 66 KB
    if (lds > 64 * 1024) {
      const int e = (int)hipFuncSetAttribute(reinterpret_cast<const void*>(pg_softmax_rows_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e) return record_hip_error(e);
    }
    hipLaunchKernelGGL(pg_softmax_rows_kernel, dim3((steps + 255) / 256), dim3(256), lds, (hipStream_t)hip_stream,
                       logits, action, discounted, probs, bottom_diff, steps, actions, make_magic((uint32_t)actions));
  } else {
    hipLaunchKernelGGL(pg_softmax_wide_kernel, dim3((steps + 3) / 4), dim3(256), 0, (hipStream_t)hip_stream, logits,
                       action, discounted, probs, bottom_diff, steps, actions);
  }
  return done();
}

}  // extern "C"
