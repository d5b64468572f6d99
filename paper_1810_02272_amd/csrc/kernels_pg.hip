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
// Four consecutive steps per thread (16-byte loads and stores); the last, partial group of a
// launch goes element by element.
__global__ __launch_bounds__(256) void pg_sample_kernel(const float* __restrict__ aprob,
                                                        const float* __restrict__ random, int32_t* __restrict__ action,
                                                        int steps) {
  const int t = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (t + 3 < steps) {
    const float4 ap = *reinterpret_cast<const float4*>(aprob + t);
    const float4 rn = *reinterpret_cast<const float4*>(random + t);
    *reinterpret_cast<int4*>(action + t) =
        make_int4(rn.x < ap.x ? 0 : 1, rn.y < ap.y ? 0 : 1, rn.z < ap.z ? 0 : 1, rn.w < ap.w ? 0 : 1);
  } else {
    for (int i = t; i < steps; ++i) action[i] = random[i] < aprob[i] ? 0 : 1;
  }
}

// ---- step 9: R[t] = reward[t] + gamma * R[t+1] inside each episode ----
// One wave per episode at a time, walking it from its end in chunks of 256 steps: lane l holds the
// four consecutive steps 4l .. 4l+3 of the chunk (one 16-byte access on a 4-byte boundary; lanes at
// the edges of the episode go element by element).  A lane first runs the recurrence over its own
// four steps; the lane totals then form the same recurrence with gamma^4 per lane, a weighted
// suffix sum: four DPP row shifts with the weights (gamma^4)^1, ^2, ^4, ^8 finish each row of 16
// lanes, three lane reads chain the rows, and the value carried in from the later chunk is added
// with the weight (gamma^4)^(64 - lane).  Each step's result is its in-lane partial plus
// gamma^(4-j) times the total of the next lane.  The scans of the chunks that are loaded together
// are independent; only the carry links them.  A wave walks several episodes with the next one's
// loads already in flight.
constexpr int kChunksInFlight = 2;
constexpr int kChunkSteps = 256;

struct Quad {
  float v[4];
};
struct __attribute__((packed, aligned(4))) QuadMem {
  float v[4];
};

// Lane l receives the value of lane l + N of its row of 16 lanes, 0 past the row's end.
template <int N>
__device__ __forceinline__ float row_shift_down(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x100 + N, 0xF, 0xF, true));
}

struct ScanWeights {
  float g1, g2, g4, g8, g16;  // powers of the per-lane factor
  float to_row_end;           // factor^(16 - lane % 16): from this lane to the first lane of the next row
  float to_chunk_end;         // factor^(64 - lane): from this lane to the first lane of the later chunk
};

__device__ __forceinline__ ScanWeights scan_weights(float factor, int lane) {
  ScanWeights w;
  w.g1 = factor;
  w.g2 = w.g1 * w.g1;
  w.g4 = w.g2 * w.g2;
  w.g8 = w.g4 * w.g4;
  w.g16 = w.g8 * w.g8;
  const int li = lane & 15;
  float p = 1.f;
  p *= (16 - li) & 1 ? w.g1 : 1.f;
  p *= (16 - li) & 2 ? w.g2 : 1.f;
  p *= (16 - li) & 4 ? w.g4 : 1.f;
  p *= (16 - li) & 8 ? w.g8 : 1.f;
  p *= (16 - li) & 16 ? w.g16 : 1.f;
  w.to_row_end = p;
  const int rows_after = 3 - (lane >> 4);
  float q = p;
  q *= rows_after & 1 ? w.g16 : 1.f;
  q *= rows_after & 2 ? w.g16 * w.g16 : 1.f;
  w.to_chunk_end = q;
  return w;
}

// v[l] <- sum over the lanes m >= l of the wave of factor^(m - l) * v[m]; t16/t32/t48 return the
// finished values of lanes 16, 32, 48 (the row heads) without the carry of a later chunk.
__device__ __forceinline__ float suffix_scan(float v, int lane, const ScanWeights& w, float& t1, float& t2, float& t3) {
  v += w.g1 * row_shift_down<1>(v);
  v += w.g2 * row_shift_down<2>(v);
  v += w.g4 * row_shift_down<4>(v);
  v += w.g8 * row_shift_down<8>(v);
  const int iv = __builtin_bit_cast(int, v);
  t3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 48));
  t2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 32)) + w.g16 * t3;
  t1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(iv, 16)) + w.g16 * t2;
  const int row = lane >> 4;
  const float later_rows = row == 0 ? t1 : row == 1 ? t2 : row == 2 ? t3 : 0.f;
  return v + w.to_row_end * later_rows;
}

__global__ __launch_bounds__(256) void pg_discount_kernel(const float* __restrict__ reward,
                                                          const int32_t* __restrict__ offsets, int episodes,
                                                          int steps, float gamma, float* __restrict__ discounted) {
  const int lane = threadIdx.x & 63;
  const int stride = (int)gridDim.x * 4;  // waves in the grid: a wave takes episodes e, e + stride, ...
  int e = (int)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
  if (e >= episodes) return;
  const float g2 = gamma * gamma, g3 = g2 * gamma, g4 = g2 * g2;
  const ScanWeights w = scan_weights(g4, lane);
  const int row = lane >> 4;

  auto bounds = [&](int ep, int& b, int& end) {  // clamped to [0, steps]; empty for ep >= episodes
    b = end = 0;
    if (ep < episodes) {
      b = offsets[ep];
      end = offsets[ep + 1];
      b = b < 0 ? 0 : (b > steps ? steps : b);
      end = end < b ? b : (end > steps ? steps : end);
    }
  };
  auto fetch = [&](Quad(&r)[kChunksInFlight], int b, int hi, int end) {  // the chunks below hi
#pragma unroll
    for (int c = 0; c < kChunksInFlight; ++c) {
      const int t = hi - kChunkSteps * (c + 1) + 4 * lane;
      if (t >= b && t + 3 < end) {
        const QuadMem m = *reinterpret_cast<const QuadMem*>(reward + t);
#pragma unroll
        for (int j = 0; j < 4; ++j) r[c].v[j] = m.v[j];
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) r[c].v[j] = (t + j >= b && t + j < end) ? reward[t + j] : 0.f;
      }
    }
  };

  // The rewards of the wave's next episode (its last chunks) and the bounds of the one after that
  // are requested before the current episode is scanned, so that their memory latency overlaps
  // the scan.
  int b, end, nb, nend;
  bounds(e, b, end);
  bounds(e + stride, nb, nend);
  Quad r[kChunksInFlight], rn[kChunksInFlight];
  fetch(r, b, end, end);
  for (;;) {
    int nnb, nnend;
    bounds(e + 2 * stride, nnb, nnend);
    fetch(rn, nb, nend, nend);
    float carry = 0.f;  // R of the first step of the later chunk
    for (int hi = end; hi > b; hi -= kChunkSteps * kChunksInFlight) {
      if (hi != end) fetch(r, b, hi, end);  // long episodes: further rounds
      float s[kChunksInFlight][4], total[kChunksInFlight], t1[kChunksInFlight], t2[kChunksInFlight], t3[kChunksInFlight];
#pragma unroll
      for (int c = 0; c < kChunksInFlight; ++c) {
        s[c][3] = r[c].v[3];
        s[c][2] = r[c].v[2] + gamma * s[c][3];
        s[c][1] = r[c].v[1] + gamma * s[c][2];
        s[c][0] = r[c].v[0] + gamma * s[c][1];
        total[c] = suffix_scan(s[c][0], lane, w, t1[c], t2[c], t3[c]);
      }
#pragma unroll
      for (int c = 0; c < kChunksInFlight; ++c) {
        const int t = hi - kChunkSteps * (c + 1) + 4 * lane;
        const float with_carry = total[c] + w.to_chunk_end * carry;
        // total of the next lane (with the carry): inside a row by a shift, at a row's last lane the
        // head of the next row, at lane 63 the carry itself
        const float h1 = t1[c] + w.g16 * w.g16 * w.g16 * carry;  // lane 16: 48 lanes before the chunk's end
        const float h2 = t2[c] + w.g16 * w.g16 * carry;
        const float h3 = t3[c] + w.g16 * carry;
        float next = row_shift_down<1>(with_carry);
        if ((lane & 15) == 15) next = row == 0 ? h1 : row == 1 ? h2 : row == 2 ? h3 : carry;
        Quad out;
        out.v[0] = with_carry;
        out.v[1] = s[c][1] + g3 * next;
        out.v[2] = s[c][2] + g2 * next;
        out.v[3] = s[c][3] + gamma * next;
        if (t >= b && t + 3 < end) {
          QuadMem m;
#pragma unroll
          for (int j = 0; j < 4; ++j) m.v[j] = out.v[j];
          *reinterpret_cast<QuadMem*>(discounted + t) = m;
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (t + j >= b && t + j < end) discounted[t + j] = out.v[j];
        }
        carry = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, with_carry)));
      }
    }
    e += stride;
    if (e >= episodes) break;
    b = nb;
    end = nend;
    nb = nnb;
    nend = nnend;
#pragma unroll
    for (int c = 0; c < kChunksInFlight; ++c) r[c] = rn[c];
  }
}

// ---- Sigmoid model, steps 8, 10, 11 ----
__global__ __launch_bounds__(256) void pg_sigmoid_kernel(const float* __restrict__ aprob,
                                                         const int32_t* __restrict__ action,
                                                         const float* __restrict__ discounted,
                                                         float* __restrict__ dlogps, float* __restrict__ bottom_diff,
                                                         int steps) {
  const int t = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (t + 3 < steps) {
    const float4 ap = *reinterpret_cast<const float4*>(aprob + t);
    const int4 ac = *reinterpret_cast<const int4*>(action + t);
    float4 w = make_float4(1.f, 1.f, 1.f, 1.f);
    if (discounted) w = *reinterpret_cast<const float4*>(discounted + t);
    const float4 d = make_float4(ac.x == 0 ? 1.f - ap.x : 0.f - ap.x, ac.y == 0 ? 1.f - ap.y : 0.f - ap.y,
                                 ac.z == 0 ? 1.f - ap.z : 0.f - ap.z, ac.w == 0 ? 1.f - ap.w : 0.f - ap.w);
    if (dlogps) *reinterpret_cast<float4*>(dlogps + t) = d;
    *reinterpret_cast<float4*>(bottom_diff + t) = make_float4(-d.x * w.x, -d.y * w.y, -d.z * w.z, -d.w * w.w);
  } else {
    for (int i = t; i < steps; ++i) {
      const float ap = aprob[i];
      const float d = action[i] == 0 ? 1.f - ap : 0.f - ap;
      if (dlogps) dlogps[i] = d;
      bottom_diff[i] = -d * (discounted ? discounted[i] : 1.f);
    }
  }
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
                                                              Magic mA, bool vec_ok) {
  extern __shared__ float tile[];  // [256][A | 1], then a second copy for the gradient
  const int AP = A | 1;
  float* const ptile = tile;
  float* const dtile = tile + 256 * AP;
  const int row0 = blockIdx.x * 256;
  const int nrows = steps - row0 < 256 ? steps - row0 : 256;
  const int count = nrows * A;
  const size_t base = (size_t)row0 * A;
  // Four-element global accesses when the block's slice is a multiple of four elements and the
  // blobs are 16-byte aligned (a block's slice then starts on such a boundary too: 256*A elements
  // per block); the (row, column) of the first element comes from one division, the next three
  // follow by stepping the column.
  const bool vec = vec_ok && (count & 3) == 0;
  if (vec) {
    for (int i = threadIdx.x * 4; i < count; i += 1024) {
      const float4 v = *reinterpret_cast<const float4*>(logits + base + i);
      int r = (int)mdiv((uint32_t)i, mA), c = i - r * A;
      const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        ptile[r * AP + c] = e[q];
        if (++c == A) {
          c = 0;
          ++r;
        }
      }
    }
  } else {
    for (int i = threadIdx.x; i < count; i += 256) {
      const int r = (int)mdiv((uint32_t)i, mA);
      ptile[r * AP + (i - r * A)] = logits[base + i];
    }
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
  if (vec) {
    for (int i = threadIdx.x * 4; i < count; i += 1024) {
      int r = (int)mdiv((uint32_t)i, mA), c = i - r * A;
      float pv[4], dv[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        pv[q] = ptile[r * AP + c];
        dv[q] = dtile[r * AP + c];
        if (++c == A) {
          c = 0;
          ++r;
        }
      }
      if (probs) *reinterpret_cast<float4*>(probs + base + i) = make_float4(pv[0], pv[1], pv[2], pv[3]);
      *reinterpret_cast<float4*>(bottom_diff + base + i) = make_float4(dv[0], dv[1], dv[2], dv[3]);
    }
  } else {
    for (int i = threadIdx.x; i < count; i += 256) {
      const int r = (int)mdiv((uint32_t)i, mA);
      const int o = r * AP + (i - r * A);
      if (probs) probs[base + i] = ptile[o];
      bottom_diff[base + i] = dtile[o];
    }
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

constexpr int32_t kMaxSteps = 0x7FFF0000;  // index arithmetic of the kernels stays below 2^31

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
  if (steps > kMaxSteps) return CONV_ESHAPE;
  if (steps == 0) return CONV_OK;
  if (!aprob || !random || !action) return CONV_EINVAL;
  hipLaunchKernelGGL(pg_sample_kernel, dim3((steps + 1023) / 1024), dim3(256), 0, (hipStream_t)hip_stream, aprob,
                     random, action, steps);
  return done();
}

int pg_discount_rewards(const float* reward, const int32_t* episode_offsets, int32_t episodes, int32_t steps,
                        float gamma, float* discounted, void* hip_stream) {
  if (episodes < 0 || steps < 0) return CONV_EINVAL;
  if (steps > kMaxSteps || episodes > kMaxSteps) return CONV_ESHAPE;
  if (episodes == 0 || steps == 0) return CONV_OK;
  if (!reward || !episode_offsets || !discounted) return CONV_EINVAL;
  int blocks = (episodes + 3) / 4;
  if (blocks > 256 * 8) blocks = 256 * 8;  // eight resident workgroups on each of the 256 compute units
  hipLaunchKernelGGL(pg_discount_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, reward,
                     episode_offsets, episodes, steps, gamma, discounted);
  return done();
}

int pg_sigmoid_bottom_diff(const float* aprob, const int32_t* action, const float* discounted, float* dlogps,
                           float* bottom_diff, int32_t steps, void* hip_stream) {
  if (steps < 0) return CONV_EINVAL;
  if (steps > kMaxSteps) return CONV_ESHAPE;
  if (steps == 0) return CONV_OK;
  if (!aprob || !action || !bottom_diff) return CONV_EINVAL;
  hipLaunchKernelGGL(pg_sigmoid_kernel, dim3((steps + 1023) / 1024), dim3(256), 0, (hipStream_t)hip_stream, aprob,
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
    static LdsOptIn opt_in;  // 32 actions need 66 KB: opt in to the largest size, once per process
    if (lds > 64 * 1024) {
      const int e = lds_opt_in(opt_in, pg_softmax_rows_kernel, 2 * 256 * 33 * (int)sizeof(float));
      if (e) return record_hip_error(e);
    }
    const bool vec_ok = (((uintptr_t)logits | (uintptr_t)probs | (uintptr_t)bottom_diff) & 15u) == 0;
    hipLaunchKernelGGL(pg_softmax_rows_kernel, dim3((steps + 255) / 256), dim3(256), lds, (hipStream_t)hip_stream,
                       logits, action, discounted, probs, bottom_diff, steps, actions, make_magic((uint32_t)actions),
                       vec_ok);
  } else {
    hipLaunchKernelGGL(pg_softmax_wide_kernel, dim3((steps + 3) / 4), dim3(256), 0, (hipStream_t)hip_stream, logits,
                       action, discounted, probs, bottom_diff, steps, actions);
  }
  return done();
}

}  // extern "C"
