// Direct kernels for thin groups (depthwise convolution and its neighbours): one thread per
// output element for forward and backward data, one lane per (position, tap) for the filter
// gradient.  No matrix unit: a group's GEMM would have one to a few rows and a handful of reduction
// indices, and the work is bound by memory, not arithmetic.  The definitions are the layer's own
// (cross-correlation, zero padding, stride, dilation, contiguous channel groups), written out per
// element; T is the base type of the blobs.
#include <hip/hip_runtime.h>
#include <stdio.h>

#include "device_utils.h"
#include "internal.h"

namespace mi355conv {
namespace {

// Consecutive workgroups go to the eight XCDs in turn; the element index is taken from the
// renumbered workgroup id so that neighbouring rows of an image, which share halo rows of the
// input, meet in one XCD's L2.
// The loops over taps are branch-free -- an element outside the image is read from a clamped
// address and multiplied by a zero weight -- so that the loads of all taps are in flight together;
// KH x KW = 0 x 0 stands for a kernel size only known at run time.

// y[n][k][oh][ow] = bias[k] + sum over the group's channels c and taps (i, j) of
//   w[k][c][i][j] * x[n][g*Cg + c][oh*sh - ph + i*dh][ow*sw - pw + j*dw]   (0 outside the image)
template <typename T, int KH, int KW>
__global__ __launch_bounds__(256) void direct_fwd_kernel(const DirectArgs a) {
  const uint32_t idx = xcd_contiguous_block_id() * 256u + threadIdx.x;
  if (idx >= a.y_elems) return;
  const int kh = KH ? KH : a.kh, kw = KW ? KW : a.kw;
  const uint32_t q1 = mdiv(idx, a.mOW), ow = idx - q1 * (uint32_t)a.OW;
  const uint32_t q2 = mdiv(q1, a.mOH), oh = q1 - q2 * (uint32_t)a.OH;
  const uint32_t n = mdiv(q2, a.mK), k = q2 - n * (uint32_t)a.K;
  const uint32_t g = mdiv(k, a.mKg);
  const T* x = static_cast<const T*>(a.in) + (n * (uint32_t)a.C + g * (uint32_t)a.Cg) * (uint32_t)(a.H * a.W);
  const T* w = static_cast<const T*>(a.w) + k * (uint32_t)(a.Cg * kh * kw);
  const int ih0 = (int)oh * a.sh - a.ph, iw0 = (int)ow * a.sw - a.pw;
  T acc = T(0);
  for (int c = 0; c < a.Cg; ++c) {
#pragma unroll
    for (int i = 0; i < kh; ++i) {
      const int ih = ih0 + i * a.dh;
      const bool row_ok = (uint32_t)ih < (uint32_t)a.H;
      const T* xr = x + (c * a.H + (row_ok ? ih : 0)) * a.W;
      const T* wr = w + (c * kh + i) * kw;
#pragma unroll
      for (int j = 0; j < kw; ++j) {
        const int iw = iw0 + j * a.dw;
        const bool ok = row_ok & ((uint32_t)iw < (uint32_t)a.W);
        acc += (ok ? wr[j] : T(0)) * xr[ok ? iw : 0];
      }
    }
  }
  if (a.bias) acc += static_cast<const T*>(a.bias)[k];
  static_cast<T*>(a.out)[idx] = acc;
}

// dx[n][c][h][w] = sum over the group's output channels k and the taps (i, j) with
//   h + ph - i*dh = sh*oh and w + pw - j*dw = sw*ow for an output position (oh, ow) of
//   w[k][c - g*Cg][i][j] * dy[n][k][oh][ow]
template <typename T, int KH, int KW>
__global__ __launch_bounds__(256) void direct_bwd_data_kernel(const DirectArgs a) {
  const uint32_t idx = xcd_contiguous_block_id() * 256u + threadIdx.x;
  if (idx >= a.x_elems) return;
  const int kh = KH ? KH : a.kh, kw = KW ? KW : a.kw;
  const uint32_t q1 = mdiv(idx, a.mW), wi = idx - q1 * (uint32_t)a.W;
  const uint32_t q2 = mdiv(q1, a.mH), hi = q1 - q2 * (uint32_t)a.H;
  const uint32_t n = mdiv(q2, a.mC), c = q2 - n * (uint32_t)a.C;
  const uint32_t g = mdiv(c, a.mCg), cl = c - g * (uint32_t)a.Cg;
  const uint32_t P = (uint32_t)(a.OH * a.OW), taps = (uint32_t)(kh * kw);
  const T* dy = static_cast<const T*>(a.in) + (n * (uint32_t)a.K + g * (uint32_t)a.Kg) * P;
  const T* w = static_cast<const T*>(a.w) + (g * (uint32_t)a.Kg * (uint32_t)a.Cg + cl) * taps;
  T acc = T(0);
  for (int k = 0; k < a.Kg; ++k) {
    const T* wk = w + (uint32_t)k * (uint32_t)a.Cg * taps;
    const T* dk = dy + (uint32_t)k * P;
#pragma unroll
    for (int i = 0; i < kh; ++i) {
      const int hh = (int)hi + a.ph - i * a.dh;
      const uint32_t oh = mdiv((uint32_t)(hh < 0 ? 0 : hh), a.mSh);
      const bool row_ok = (hh >= 0) & (oh * (uint32_t)a.sh == (uint32_t)hh) & (oh < (uint32_t)a.OH);
      const T* dr = dk + (row_ok ? oh : 0u) * (uint32_t)a.OW;
#pragma unroll
      for (int j = 0; j < kw; ++j) {
        const int ww = (int)wi + a.pw - j * a.dw;
        const uint32_t ow = mdiv((uint32_t)(ww < 0 ? 0 : ww), a.mSw);
        const bool ok = row_ok & (ww >= 0) & (ow * (uint32_t)a.sw == (uint32_t)ww) & (ow < (uint32_t)a.OW);
        acc += (ok ? wk[i * kw + j] : T(0)) * dr[ok ? ow : 0u];
      }
    }
  }
  static_cast<T*>(a.out)[idx] = acc;
}

// Sum of v over the 64 lanes of a wave, in a fixed order; lane 0 stores it.
template <typename T>
__device__ __forceinline__ void wave_sum_to(T v, int lane, T* dst) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_down(v, off, 64);
  if (lane == 0) *dst = v;
}

// part[s][k][c][i][j] = sum over the images of split s and all output positions of
//   dy[n][k][oh][ow] * x[n][g*Cg + c][oh*sh - ph + i*dh][ow*sw - pw + j*dw]
// One workgroup per ((k, c) pair, split).  Lane l of a wave stands for tap l % taps of position
// slot l / taps, so an iteration of a wave covers `slots` consecutive output positions of one image
// with every tap (one load of dy, broadcast over the taps, and one load of x per lane); the four
// waves take the (image, chunk of positions) units in turn, four units in flight per wave.  The
// per-lane sums are added over slots and waves in a fixed order.
// With a.bias_part set, the workgroups of a group's first input channel (c == 0) also add up the dy
// values they read -- each exactly once -- and store bias_part[s][k]: the bias gradient's share of
// split s, finished by the reduce kernel together with the filter gradient.  The same holds for the
// 3x3 / 5x5 filter-gradient kernels below.
template <typename T>
__global__ __launch_bounds__(256) void direct_wgrad_kernel(const DirectArgs a) {
  __shared__ T red[256];
  constexpr int kInFlight = 4;
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  const uint32_t pair = blockIdx.x, split = blockIdx.y;
  const uint32_t k = mdiv(pair, a.mCg), c = pair - k * (uint32_t)a.Cg;
  const uint32_t g = mdiv(k, a.mKg);
  const uint32_t slot = mdiv((uint32_t)lane, a.mTaps), tap = (uint32_t)lane - slot * (uint32_t)a.taps;
  const uint32_t ti = mdiv(tap, a.mKw), tj = tap - ti * (uint32_t)a.kw;
  const bool lane_on = slot < (uint32_t)a.slots;
  const int dih = (int)ti * a.dh - a.ph, diw = (int)tj * a.dw - a.pw;
  const uint32_t P = (uint32_t)(a.OH * a.OW), HW = (uint32_t)(a.H * a.W);
  const uint32_t n0 = split * (uint32_t)a.imgs_per_split;
  const uint32_t n1 = n0 + (uint32_t)a.imgs_per_split < (uint32_t)a.N ? n0 + (uint32_t)a.imgs_per_split : (uint32_t)a.N;
  const uint32_t units = (n1 - n0) * (uint32_t)a.chunks_per_img;
  const T* dy = static_cast<const T*>(a.w) + k * P;                                        // + n*K*P + pos
  const T* x = static_cast<const T*>(a.in) + (g * (uint32_t)a.Cg + c) * HW;                // + n*C*HW + ih*W + iw
  T acc = T(0);
  const bool row_sum = a.bias_part != nullptr && c == 0;  // uniform over the workgroup
  T bsum = T(0);
  for (uint32_t u0 = (uint32_t)wv; u0 < units; u0 += 4 * kInFlight) {
    T dv[kInFlight], xv[kInFlight];
#pragma unroll
    for (int q = 0; q < kInFlight; ++q) {
      const uint32_t u = u0 + 4u * (uint32_t)q;
      const uint32_t nl = mdiv(u, a.mChunks), ch = u - nl * (uint32_t)a.chunks_per_img;
      const uint32_t pos = ch * (uint32_t)a.slots + slot;
      const uint32_t oh = mdiv(pos, a.mOW), ow = pos - oh * (uint32_t)a.OW;
      const int ih = (int)oh * a.sh + dih, iw = (int)ow * a.sw + diw;
      const bool okd = lane_on & (u < units) & (pos < P);  // a real element of dy
      const bool ok = okd & ((uint32_t)ih < (uint32_t)a.H) & ((uint32_t)iw < (uint32_t)a.W);
      const uint32_t n = n0 + nl;
      const T d = dy[okd ? n * (uint32_t)a.K * P + pos : 0u];
      dv[q] = ok ? d : T(0);
      if (row_sum) bsum += (okd && tap == 0) ? d : T(0);  // every element of dy once: the lanes of tap 0
      xv[q] = x[ok ? n * (uint32_t)a.C * HW + (uint32_t)ih * (uint32_t)a.W + (uint32_t)iw : 0u];
    }
#pragma unroll
    for (int q = 0; q < kInFlight; ++q) acc += dv[q] * xv[q];
  }
  red[t] = acc;
  __shared__ T bred[4];
  if (row_sum) wave_sum_to(bsum, lane, &bred[wv]);
  __syncthreads();
  if (t < a.taps) {
    T sum = T(0);
    for (int w4 = 0; w4 < 4; ++w4)
      for (int sl = 0; sl < a.slots; ++sl) sum += red[w4 * 64 + sl * a.taps + t];
    static_cast<T*>(a.part)[split * a.w_elems + pair * (uint32_t)a.taps + (uint32_t)t] = sum;
  }
  if (row_sum && t == 0)
    static_cast<T*>(a.bias_part)[split * (uint32_t)a.K + k] = ((bred[0] + bred[1]) + bred[2]) + bred[3];
}

// ---- 3x3 and 5x5 kernels: several output rows per thread ----
// A thread owns output rows R*ohb .. R*ohb+R-1 of one column: the weights of a channel are read once
// for all of them, and with unit stride and dilation (UNIT) the R + KH - 1 input rows they touch
// are read once instead of KH times.  FLIP reverses the taps: backward data of a stride-1
// layer is the forward pass of the mirrored kernel with the roles of the blobs exchanged (the host
// code swaps the fields and sets the padding to dilation*(k-1) - pad, which may be negative).
// Rows per thread: eight where the input rows are shared between them, four where every tap of every
// row is a load of its own.
constexpr int rows_per_thread(bool unit) { return unit ? 8 : 4; }

template <typename T, int KH, int KW, bool UNIT>
__device__ __forceinline__ void load_window(const DirectArgs& a, const T* xc, int oh0, int ow,
                                            T (&xs)[rows_per_thread(UNIT) + KH - 1][KW]) {
  static_assert(UNIT, "window form needs unit stride and dilation");
  constexpr int kRows = rows_per_thread(UNIT);
#pragma unroll
  for (int rr = 0; rr < kRows + KH - 1; ++rr) {
    const int ih = oh0 - a.ph + rr;
    const bool row_ok = (uint32_t)ih < (uint32_t)a.H;
    const T* xr = xc + (row_ok ? ih : 0) * a.W;
#pragma unroll
    for (int j = 0; j < KW; ++j) {
      const int iw = ow - a.pw + j;
      const bool ok = row_ok & ((uint32_t)iw < (uint32_t)a.W);
      const T v = xr[ok ? iw : 0];
      xs[rr][j] = ok ? v : T(0);
    }
  }
}

template <typename T>
__device__ __forceinline__ T load_tap(const DirectArgs& a, const T* xc, int ih, int iw) {
  const bool ok = ((uint32_t)ih < (uint32_t)a.H) & ((uint32_t)iw < (uint32_t)a.W);
  const T v = xc[ok ? ih * a.W + iw : 0];
  return ok ? v : T(0);
}

template <typename T, int KH, int KW, bool UNIT, bool FLIP>
__global__ __launch_bounds__(256) void direct_rows_kernel(const DirectArgs a) {
  constexpr int kRows = rows_per_thread(UNIT);
  const uint32_t idx = xcd_contiguous_block_id() * 256u + threadIdx.x;
  if (idx >= a.row_items) return;
  const uint32_t q1 = mdiv(idx, a.mOW), ow = idx - q1 * (uint32_t)a.OW;
  const uint32_t q2 = mdiv(q1, a.mOHB), ohb = q1 - q2 * (uint32_t)a.OHB;
  const uint32_t n = mdiv(q2, a.mK), k = q2 - n * (uint32_t)a.K;
  const uint32_t g = mdiv(k, a.mKg), kl = k - g * (uint32_t)a.Kg;
  const uint32_t HW = (uint32_t)(a.H * a.W);
  const T* x = static_cast<const T*>(a.in) + (n * (uint32_t)a.C + g * (uint32_t)a.Cg) * HW;
  const T* w = static_cast<const T*>(a.w) + g * (uint32_t)(a.Kg * a.Cg * KH * KW) + kl * a.w_out_stride;
  const int oh0 = (int)ohb * kRows;
  T acc[kRows];
#pragma unroll
  for (int r = 0; r < kRows; ++r) acc[r] = T(0);
  for (int c = 0; c < a.Cg; ++c) {
    T wv[KH][KW];
#pragma unroll
    for (int i = 0; i < KH; ++i)
#pragma unroll
      for (int j = 0; j < KW; ++j)
        wv[i][j] = w[(uint32_t)c * a.w_in_stride + (uint32_t)(FLIP ? (KH - 1 - i) * KW + (KW - 1 - j) : i * KW + j)];
    const T* xc = x + (uint32_t)c * HW;
    if constexpr (UNIT) {
      T xs[kRows + KH - 1][KW];
      load_window<T, KH, KW, UNIT>(a, xc, oh0, (int)ow, xs);
#pragma unroll
      for (int r = 0; r < kRows; ++r)
#pragma unroll
        for (int i = 0; i < KH; ++i)
#pragma unroll
          for (int j = 0; j < KW; ++j) acc[r] += wv[i][j] * xs[r + i][j];
    } else {
#pragma unroll
      for (int r = 0; r < kRows; ++r)
#pragma unroll
        for (int i = 0; i < KH; ++i)
#pragma unroll
          for (int j = 0; j < KW; ++j)
            acc[r] += wv[i][j] * load_tap(a, xc, (oh0 + r) * a.sh - a.ph + i * a.dh, (int)ow * a.sw - a.pw + j * a.dw);
    }
  }
  const T bb = a.bias ? static_cast<const T*>(a.bias)[k] : T(0);
  T* out = static_cast<T*>(a.out) + ((n * (uint32_t)a.K + k) * (uint32_t)a.OH + (uint32_t)oh0) * (uint32_t)a.OW + ow;
#pragma unroll
  for (int r = 0; r < kRows; ++r)
    if (oh0 + r < a.OH) {
      out[(uint32_t)r * (uint32_t)a.OW] = acc[r] + bb;
    }
}

// ---- "same" convolutions with rows of a multiple of four elements: four columns per thread ----
// Unit stride and dilation, pad_w = (KW-1)/2 (so OW = W), W a multiple of 4 and 16-byte aligned
// blobs: a thread owns a 4-row x 4-column block of the output.  Each input row of its window is
// one aligned four-element load plus (KW-1)/2 halo elements on either side, and the outputs leave
// as four-element stores -- a quarter of the memory instructions of the one-column form.
constexpr int kVecRows = 4, kVecCols = 4;

template <typename T>
struct alignas(4 * sizeof(T)) Vec4 {
  T v[4];
};

template <typename T, int KH, int KW>
__device__ __forceinline__ void load_window_vec(const DirectArgs& a, const T* xc, int oh0, int ow0,
                                                T (&xs)[kVecRows + KH - 1][kVecCols + KW - 1]) {
  constexpr int PW = (KW - 1) / 2;
#pragma unroll
  for (int rr = 0; rr < kVecRows + KH - 1; ++rr) {
    const int ih = oh0 - a.ph + rr;
    const bool row_ok = (uint32_t)ih < (uint32_t)a.H;
    const T* xr = xc + (row_ok ? ih : 0) * a.W;
    const Vec4<T> mid = *reinterpret_cast<const Vec4<T>*>(xr + ow0);
#pragma unroll
    for (int v = 0; v < kVecCols; ++v) xs[rr][PW + v] = row_ok ? mid.v[v] : T(0);
#pragma unroll
    for (int j = 0; j < PW; ++j) {
      const int il = ow0 - PW + j, ir = ow0 + kVecCols + j;
      const bool okl = row_ok & (il >= 0), okr = row_ok & (ir < a.W);
      const T vl = xr[okl ? il : 0], vr = xr[okr ? ir : 0];
      xs[rr][j] = okl ? vl : T(0);
      xs[rr][PW + kVecCols + j] = okr ? vr : T(0);
    }
  }
}

template <typename T, int KH, int KW, bool FLIP>
__global__ __launch_bounds__(256) void direct_rows_vec_kernel(const DirectArgs a) {
  const uint32_t idx = xcd_contiguous_block_id() * 256u + threadIdx.x;
  if (idx >= a.row_items) return;
  const uint32_t q1 = mdiv(idx, a.mOWQ), owq = idx - q1 * (uint32_t)a.OWQ;
  const uint32_t q2 = mdiv(q1, a.mOHB), ohb = q1 - q2 * (uint32_t)a.OHB;
  const uint32_t n = mdiv(q2, a.mK), k = q2 - n * (uint32_t)a.K;
  const uint32_t g = mdiv(k, a.mKg), kl = k - g * (uint32_t)a.Kg;
  const uint32_t HW = (uint32_t)(a.H * a.W);
  const T* x = static_cast<const T*>(a.in) + (n * (uint32_t)a.C + g * (uint32_t)a.Cg) * HW;
  const T* w = static_cast<const T*>(a.w) + g * (uint32_t)(a.Kg * a.Cg * KH * KW) + kl * a.w_out_stride;
  const int oh0 = (int)ohb * kVecRows, ow0 = (int)owq * kVecCols;
  T acc[kVecRows][kVecCols];
#pragma unroll
  for (int r = 0; r < kVecRows; ++r)
#pragma unroll
    for (int v = 0; v < kVecCols; ++v) acc[r][v] = T(0);
  for (int c = 0; c < a.Cg; ++c) {
    T wv[KH][KW];
#pragma unroll
    for (int i = 0; i < KH; ++i)
#pragma unroll
      for (int j = 0; j < KW; ++j)
        wv[i][j] = w[(uint32_t)c * a.w_in_stride + (uint32_t)(FLIP ? (KH - 1 - i) * KW + (KW - 1 - j) : i * KW + j)];
    T xs[kVecRows + KH - 1][kVecCols + KW - 1];
    load_window_vec<T, KH, KW>(a, x + (uint32_t)c * HW, oh0, ow0, xs);
#pragma unroll
    for (int r = 0; r < kVecRows; ++r)
#pragma unroll
      for (int i = 0; i < KH; ++i)
#pragma unroll
        for (int j = 0; j < KW; ++j)
#pragma unroll
          for (int v = 0; v < kVecCols; ++v) acc[r][v] += wv[i][j] * xs[r + i][v + j];
  }
  const T bb = a.bias ? static_cast<const T*>(a.bias)[k] : T(0);
  T* out = static_cast<T*>(a.out) + ((n * (uint32_t)a.K + k) * (uint32_t)a.OH + (uint32_t)oh0) * (uint32_t)a.OW + (uint32_t)ow0;
#pragma unroll
  for (int r = 0; r < kVecRows; ++r)
    if (oh0 + r < a.OH) {
      Vec4<T>* dst = reinterpret_cast<Vec4<T>*>(out + (uint32_t)r * (uint32_t)a.OW);
      Vec4<T> o;
#pragma unroll
      for (int v = 0; v < kVecCols; ++v) o.v[v] = acc[r][v] + bb;
      *dst = o;
    }
}

template <typename T, int KH, int KW>
__global__ __launch_bounds__(256) void direct_wgrad_rows_vec_kernel(const DirectArgs a) {
  __shared__ T red[4][KH * KW];
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  const uint32_t pair = blockIdx.x, split = blockIdx.y;
  const uint32_t k = mdiv(pair, a.mCg), c = pair - k * (uint32_t)a.Cg;
  const uint32_t g = mdiv(k, a.mKg);
  const uint32_t P = (uint32_t)(a.OH * a.OW), HW = (uint32_t)(a.H * a.W);
  const uint32_t n0 = split * (uint32_t)a.imgs_per_split;
  const uint32_t n1 = n0 + (uint32_t)a.imgs_per_split < (uint32_t)a.N ? n0 + (uint32_t)a.imgs_per_split : (uint32_t)a.N;
  const uint32_t items = (n1 - n0) * (uint32_t)a.OHB * (uint32_t)a.OWQ;
  const T* dy = static_cast<const T*>(a.w) + k * P;
  const T* x = static_cast<const T*>(a.in) + (g * (uint32_t)a.Cg + c) * HW;
  T acc[KH][KW];
#pragma unroll
  for (int i = 0; i < KH; ++i)
#pragma unroll
    for (int j = 0; j < KW; ++j) acc[i][j] = T(0);
  const bool row_sum = a.bias_part != nullptr && c == 0;  // uniform over the workgroup
  T bsum = T(0);
  __shared__ T bred[4];
  for (uint32_t item = (uint32_t)t; item < items; item += 256u) {
    const uint32_t q1 = mdiv(item, a.mOWQ), owq = item - q1 * (uint32_t)a.OWQ;
    const uint32_t nl = mdiv(q1, a.mOHB), ohb = q1 - nl * (uint32_t)a.OHB;
    const uint32_t n = n0 + nl;
    const int oh0 = (int)ohb * kVecRows, ow0 = (int)owq * kVecCols;
    const T* dn = dy + n * (uint32_t)a.K * P + (uint32_t)ow0;
    T dv[kVecRows][kVecCols];
#pragma unroll
    for (int r = 0; r < kVecRows; ++r) {
      const bool ok = oh0 + r < a.OH;
      const Vec4<T> d4 = *reinterpret_cast<const Vec4<T>*>(dn + (ok ? (uint32_t)(oh0 + r) * (uint32_t)a.OW : 0u));
#pragma unroll
      for (int v = 0; v < kVecCols; ++v) dv[r][v] = ok ? d4.v[v] : T(0);
    }
    if (row_sum) {
#pragma unroll
      for (int r = 0; r < kVecRows; ++r) bsum += (dv[r][0] + dv[r][1]) + (dv[r][2] + dv[r][3]);
    }
    T xs[kVecRows + KH - 1][kVecCols + KW - 1];
    load_window_vec<T, KH, KW>(a, x + n * (uint32_t)a.C * HW, oh0, ow0, xs);
#pragma unroll
    for (int i = 0; i < KH; ++i)
#pragma unroll
      for (int j = 0; j < KW; ++j)
#pragma unroll
        for (int r = 0; r < kVecRows; ++r)
#pragma unroll
          for (int v = 0; v < kVecCols; ++v) acc[i][j] += dv[r][v] * xs[r + i][v + j];
  }
#pragma unroll
  for (int i = 0; i < KH; ++i)
#pragma unroll
    for (int j = 0; j < KW; ++j) {
      T v = acc[i][j];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) v += __shfl_down(v, off, 64);
      if (lane == 0) red[wv][i * KW + j] = v;
    }
  if (row_sum) wave_sum_to(bsum, lane, &bred[wv]);
  __syncthreads();
  if (t < KH * KW)
    static_cast<T*>(a.part)[split * a.w_elems + pair * (uint32_t)(KH * KW) + (uint32_t)t] =
        ((red[0][t] + red[1][t]) + red[2][t]) + red[3][t];
  if (row_sum && t == 0)
    static_cast<T*>(a.bias_part)[split * (uint32_t)a.K + k] = ((bred[0] + bred[1]) + bred[2]) + bred[3];
}

// ---- stride 2, "same" padding along rows of a multiple of four elements ----
// A thread owns four output rows x two output columns (2q, 2q+1): their windows span the input
// columns 4q - pad_w .. 4q + KW - pad_w + 1, i.e. one aligned four-element load per input row plus
// the halo elements, and the two outputs of a row leave as one two-element store.
constexpr int kS2Rows = 4, kS2Cols = 2;

template <typename T>
struct alignas(2 * sizeof(T)) Vec2 {
  T v[2];
};

template <typename T, int KH, int KW>
__device__ __forceinline__ void load_window_s2(const DirectArgs& a, const T* xc, int oh0, int q,
                                               T (&xs)[2 * (kS2Rows - 1) + KH][KW + 2]) {
  constexpr int PW = (KW - 1) / 2, RIGHT = KW - 2 - PW;
#pragma unroll
  for (int rr = 0; rr < 2 * (kS2Rows - 1) + KH; ++rr) {
    const int ih = 2 * oh0 - a.ph + rr;
    const bool row_ok = (uint32_t)ih < (uint32_t)a.H;
    const T* xr = xc + (row_ok ? ih : 0) * a.W;
    const Vec4<T> mid = *reinterpret_cast<const Vec4<T>*>(xr + 4 * q);
#pragma unroll
    for (int v = 0; v < 4; ++v) xs[rr][PW + v] = row_ok ? mid.v[v] : T(0);
#pragma unroll
    for (int j = 0; j < PW; ++j) {
      const int il = 4 * q - PW + j;
      const bool ok = row_ok & (il >= 0);
      const T v = xr[ok ? il : 0];
      xs[rr][j] = ok ? v : T(0);
    }
#pragma unroll
    for (int j = 0; j < RIGHT; ++j) {
      const int ir = 4 * q + 4 + j;
      const bool ok = row_ok & (ir < a.W);
      const T v = xr[ok ? ir : 0];
      xs[rr][PW + 4 + j] = ok ? v : T(0);
    }
  }
}

template <typename T, int KH, int KW>
__global__ __launch_bounds__(256) void direct_rows_s2_kernel(const DirectArgs a) {
  const uint32_t idx = xcd_contiguous_block_id() * 256u + threadIdx.x;
  if (idx >= a.row_items) return;
  const uint32_t q1 = mdiv(idx, a.mOWQ), q = idx - q1 * (uint32_t)a.OWQ;
  const uint32_t q2 = mdiv(q1, a.mOHB), ohb = q1 - q2 * (uint32_t)a.OHB;
  const uint32_t n = mdiv(q2, a.mK), k = q2 - n * (uint32_t)a.K;
  const uint32_t g = mdiv(k, a.mKg), kl = k - g * (uint32_t)a.Kg;
  const uint32_t HW = (uint32_t)(a.H * a.W);
  const T* x = static_cast<const T*>(a.in) + (n * (uint32_t)a.C + g * (uint32_t)a.Cg) * HW;
  const T* w = static_cast<const T*>(a.w) + (g * (uint32_t)a.Kg + kl) * (uint32_t)(a.Cg * KH * KW);
  const int oh0 = (int)ohb * kS2Rows;
  T acc[kS2Rows][kS2Cols];
#pragma unroll
  for (int r = 0; r < kS2Rows; ++r)
#pragma unroll
    for (int v = 0; v < kS2Cols; ++v) acc[r][v] = T(0);
  for (int c = 0; c < a.Cg; ++c) {
    T wv[KH][KW];
#pragma unroll
    for (int i = 0; i < KH; ++i)
#pragma unroll
      for (int j = 0; j < KW; ++j) wv[i][j] = w[(uint32_t)(c * KH * KW + i * KW + j)];
    T xs[2 * (kS2Rows - 1) + KH][KW + 2];
    load_window_s2<T, KH, KW>(a, x + (uint32_t)c * HW, oh0, (int)q, xs);
#pragma unroll
    for (int r = 0; r < kS2Rows; ++r)
#pragma unroll
      for (int i = 0; i < KH; ++i)
#pragma unroll
        for (int j = 0; j < KW; ++j)
#pragma unroll
          for (int v = 0; v < kS2Cols; ++v) acc[r][v] += wv[i][j] * xs[2 * r + i][2 * v + j];
  }
  const T bb = a.bias ? static_cast<const T*>(a.bias)[k] : T(0);
  T* out = static_cast<T*>(a.out) + ((n * (uint32_t)a.K + k) * (uint32_t)a.OH + (uint32_t)oh0) * (uint32_t)a.OW + 2u * q;
#pragma unroll
  for (int r = 0; r < kS2Rows; ++r)
    if (oh0 + r < a.OH) {
      Vec2<T> o;
      o.v[0] = acc[r][0] + bb;
      o.v[1] = acc[r][1] + bb;
      *reinterpret_cast<Vec2<T>*>(out + (uint32_t)r * (uint32_t)a.OW) = o;
    }
}

template <typename T, int KH, int KW>
__global__ __launch_bounds__(256) void direct_wgrad_rows_s2_kernel(const DirectArgs a) {
  __shared__ T red[4][KH * KW];
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  const uint32_t pair = blockIdx.x, split = blockIdx.y;
  const uint32_t k = mdiv(pair, a.mCg), c = pair - k * (uint32_t)a.Cg;
  const uint32_t g = mdiv(k, a.mKg);
  const uint32_t P = (uint32_t)(a.OH * a.OW), HW = (uint32_t)(a.H * a.W);
  const uint32_t n0 = split * (uint32_t)a.imgs_per_split;
  const uint32_t n1 = n0 + (uint32_t)a.imgs_per_split < (uint32_t)a.N ? n0 + (uint32_t)a.imgs_per_split : (uint32_t)a.N;
  const uint32_t items = (n1 - n0) * (uint32_t)a.OHB * (uint32_t)a.OWQ;
  const T* dy = static_cast<const T*>(a.w) + k * P;
  const T* x = static_cast<const T*>(a.in) + (g * (uint32_t)a.Cg + c) * HW;
  T acc[KH][KW];
#pragma unroll
  for (int i = 0; i < KH; ++i)
#pragma unroll
    for (int j = 0; j < KW; ++j) acc[i][j] = T(0);
  const bool row_sum = a.bias_part != nullptr && c == 0;  // uniform over the workgroup
  T bsum = T(0);
  __shared__ T bred[4];
  for (uint32_t item = (uint32_t)t; item < items; item += 256u) {
    const uint32_t q1 = mdiv(item, a.mOWQ), q = item - q1 * (uint32_t)a.OWQ;
    const uint32_t nl = mdiv(q1, a.mOHB), ohb = q1 - nl * (uint32_t)a.OHB;
    const uint32_t n = n0 + nl;
    const int oh0 = (int)ohb * kS2Rows;
    const T* dn = dy + n * (uint32_t)a.K * P + 2u * q;
    T dv[kS2Rows][kS2Cols];
#pragma unroll
    for (int r = 0; r < kS2Rows; ++r) {
      const bool ok = oh0 + r < a.OH;
      const Vec2<T> d2 = *reinterpret_cast<const Vec2<T>*>(dn + (ok ? (uint32_t)(oh0 + r) * (uint32_t)a.OW : 0u));
      dv[r][0] = ok ? d2.v[0] : T(0);
      dv[r][1] = ok ? d2.v[1] : T(0);
    }
    if (row_sum) {
#pragma unroll
      for (int r = 0; r < kS2Rows; ++r) bsum += dv[r][0] + dv[r][1];
    }
    T xs[2 * (kS2Rows - 1) + KH][KW + 2];
    load_window_s2<T, KH, KW>(a, x + n * (uint32_t)a.C * HW, oh0, (int)q, xs);
#pragma unroll
    for (int i = 0; i < KH; ++i)
#pragma unroll
      for (int j = 0; j < KW; ++j)
#pragma unroll
        for (int r = 0; r < kS2Rows; ++r)
#pragma unroll
          for (int v = 0; v < kS2Cols; ++v) acc[i][j] += dv[r][v] * xs[2 * r + i][2 * v + j];
  }
#pragma unroll
  for (int i = 0; i < KH; ++i)
#pragma unroll
    for (int j = 0; j < KW; ++j) {
      T v = acc[i][j];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) v += __shfl_down(v, off, 64);
      if (lane == 0) red[wv][i * KW + j] = v;
    }
  if (row_sum) wave_sum_to(bsum, lane, &bred[wv]);
  __syncthreads();
  if (t < KH * KW)
    static_cast<T*>(a.part)[split * a.w_elems + pair * (uint32_t)(KH * KW) + (uint32_t)t] =
        ((red[0][t] + red[1][t]) + red[2][t]) + red[3][t];
  if (row_sum && t == 0)
    static_cast<T*>(a.bias_part)[split * (uint32_t)a.K + k] = ((bred[0] + bred[1]) + bred[2]) + bred[3];
}

// Stride-2 launcher for forward (pass 0) and filter gradient (pass 2); false when the shape or the
// alignment of the blobs does not fit (the caller then takes the one-column kernels).
template <typename T, int KH, int KW>
int launch_s2(int pass, const DirectArgs& src, hipStream_t s) {
  DirectArgs a = src;
  a.OWQ = src.W / 4;
  a.mOWQ = make_magic((uint32_t)a.OWQ);
  a.OHB = (a.OH + kS2Rows - 1) / kS2Rows;
  a.mOHB = make_magic((uint32_t)a.OHB);
  if (pass == 0) {
    a.row_items = (uint32_t)a.N * (uint32_t)a.K * (uint32_t)a.OHB * (uint32_t)a.OWQ;
    hipLaunchKernelGGL((direct_rows_s2_kernel<T, KH, KW>), dim3((a.row_items + 255u) / 256u), dim3(256), 0, s, a);
  } else {
    hipLaunchKernelGGL((direct_wgrad_rows_s2_kernel<T, KH, KW>), dim3((uint32_t)(a.K * a.Cg), (uint32_t)a.S), dim3(256),
                       0, s, a);
  }
  return (int)hipGetLastError();
}

// Filter gradient, 3x3 and 5x5: lanes are output columns, a thread keeps one running sum per tap
// over its (image, R rows, column) items; the sums are then added over the wave (fixed
// shuffle tree) and over the four waves.
template <typename T, int KH, int KW, bool UNIT>
__global__ __launch_bounds__(256) void direct_wgrad_rows_kernel(const DirectArgs a) {
  constexpr int kRows = rows_per_thread(UNIT);
  __shared__ T red[4][KH * KW];
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  const uint32_t pair = blockIdx.x, split = blockIdx.y;
  const uint32_t k = mdiv(pair, a.mCg), c = pair - k * (uint32_t)a.Cg;
  const uint32_t g = mdiv(k, a.mKg);
  const uint32_t P = (uint32_t)(a.OH * a.OW), HW = (uint32_t)(a.H * a.W);
  const uint32_t n0 = split * (uint32_t)a.imgs_per_split;
  const uint32_t n1 = n0 + (uint32_t)a.imgs_per_split < (uint32_t)a.N ? n0 + (uint32_t)a.imgs_per_split : (uint32_t)a.N;
  const uint32_t items = (n1 - n0) * (uint32_t)a.OHB * (uint32_t)a.OW;
  const T* dy = static_cast<const T*>(a.w) + k * P;
  const T* x = static_cast<const T*>(a.in) + (g * (uint32_t)a.Cg + c) * HW;
  T acc[KH][KW];
#pragma unroll
  for (int i = 0; i < KH; ++i)
#pragma unroll
    for (int j = 0; j < KW; ++j) acc[i][j] = T(0);
  const bool row_sum = a.bias_part != nullptr && c == 0;  // uniform over the workgroup
  T bsum = T(0);
  __shared__ T bred[4];
  for (uint32_t item = (uint32_t)t; item < items; item += 256u) {
    const uint32_t q1 = mdiv(item, a.mOW), ow = item - q1 * (uint32_t)a.OW;
    const uint32_t nl = mdiv(q1, a.mOHB), ohb = q1 - nl * (uint32_t)a.OHB;
    const uint32_t n = n0 + nl;
    const int oh0 = (int)ohb * kRows;
    const T* dn = dy + n * (uint32_t)a.K * P + ow;
    const T* xc = x + n * (uint32_t)a.C * HW;
    T dv[kRows];
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
      const bool ok = oh0 + r < a.OH;
      const T v = dn[ok ? (uint32_t)(oh0 + r) * (uint32_t)a.OW : 0u];
      dv[r] = ok ? v : T(0);
    }
    if (row_sum) {
#pragma unroll
      for (int r = 0; r < kRows; ++r) bsum += dv[r];
    }
    if constexpr (UNIT) {
      T xs[kRows + KH - 1][KW];
      load_window<T, KH, KW, UNIT>(a, xc, oh0, (int)ow, xs);
#pragma unroll
      for (int r = 0; r < kRows; ++r)
#pragma unroll
        for (int i = 0; i < KH; ++i)
#pragma unroll
          for (int j = 0; j < KW; ++j) acc[i][j] += dv[r] * xs[r + i][j];
    } else {
#pragma unroll
      for (int r = 0; r < kRows; ++r)
#pragma unroll
        for (int i = 0; i < KH; ++i)
#pragma unroll
          for (int j = 0; j < KW; ++j)
            acc[i][j] += dv[r] * load_tap(a, xc, (oh0 + r) * a.sh - a.ph + i * a.dh, (int)ow * a.sw - a.pw + j * a.dw);
    }
  }
#pragma unroll
  for (int i = 0; i < KH; ++i)
#pragma unroll
    for (int j = 0; j < KW; ++j) {
      T v = acc[i][j];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) v += __shfl_down(v, off, 64);
      if (lane == 0) red[wv][i * KW + j] = v;
    }
  if (row_sum) wave_sum_to(bsum, lane, &bred[wv]);
  __syncthreads();
  if (t < KH * KW)
    static_cast<T*>(a.part)[split * a.w_elems + pair * (uint32_t)(KH * KW) + (uint32_t)t] =
        ((red[0][t] + red[1][t]) + red[2][t]) + red[3][t];
  if (row_sum && t == 0)
    static_cast<T*>(a.bias_part)[split * (uint32_t)a.K + k] = ((bred[0] + bred[1]) + bred[2]) + bred[3];
}

// Backward data at stride S (dilation 1), 3x3 and 5x5: a thread owns the S x S block of dx with
// h + ph = S*a + rh, w + pw = S*b + rw.  Tap (i, j) reaches phase (rh, rw) exactly when i - rh and
// j - rw are non-negative multiples of S, and then reads dy at (a - (i-rh)/S, b - (j-rw)/S): the
// block needs only ((KH-1)/S + 1) x ((KW-1)/S + 1) values of dy per channel and uses every tap once.
template <typename T, int KH, int KW, int S>
__global__ __launch_bounds__(256) void direct_bwd_blocks_kernel(const DirectArgs a) {
  constexpr int QH = (KH - 1) / S + 1, QW = (KW - 1) / S + 1;
  const uint32_t idx = xcd_contiguous_block_id() * 256u + threadIdx.x;
  if (idx >= a.block_items) return;
  const uint32_t q1 = mdiv(idx, a.mBW), bb = idx - q1 * (uint32_t)a.BW;
  const uint32_t q2 = mdiv(q1, a.mBH), ba = q1 - q2 * (uint32_t)a.BH;
  const uint32_t n = mdiv(q2, a.mC), c = q2 - n * (uint32_t)a.C;
  const uint32_t g = mdiv(c, a.mCg), cl = c - g * (uint32_t)a.Cg;
  const uint32_t P = (uint32_t)(a.OH * a.OW);
  const T* dy = static_cast<const T*>(a.in) + (n * (uint32_t)a.K + g * (uint32_t)a.Kg) * P;
  const T* w = static_cast<const T*>(a.w) + (g * (uint32_t)a.Kg * (uint32_t)a.Cg + cl) * (uint32_t)(KH * KW);
  T acc[S][S];
#pragma unroll
  for (int rh = 0; rh < S; ++rh)
#pragma unroll
    for (int rw = 0; rw < S; ++rw) acc[rh][rw] = T(0);
  for (int k = 0; k < a.Kg; ++k) {
    const T* wk = w + (uint32_t)k * (uint32_t)a.Cg * (uint32_t)(KH * KW);
    const T* dk = dy + (uint32_t)k * P;
    T dv[QH][QW];
#pragma unroll
    for (int qh = 0; qh < QH; ++qh)
#pragma unroll
      for (int qw = 0; qw < QW; ++qw) {
        const int oh = (int)ba - qh, ow = (int)bb - qw;
        const bool ok = ((uint32_t)oh < (uint32_t)a.OH) & ((uint32_t)ow < (uint32_t)a.OW);
        const T v = dk[ok ? oh * a.OW + ow : 0];
        dv[qh][qw] = ok ? v : T(0);
      }
#pragma unroll
    for (int i = 0; i < KH; ++i)
#pragma unroll
      for (int j = 0; j < KW; ++j) acc[i % S][j % S] += wk[i * KW + j] * dv[i / S][j / S];
  }
#pragma unroll
  for (int rh = 0; rh < S; ++rh)
#pragma unroll
    for (int rw = 0; rw < S; ++rw) {
      const int h = (int)ba * S + rh - a.ph, wi = (int)bb * S + rw - a.pw;
      if ((uint32_t)h < (uint32_t)a.H && (uint32_t)wi < (uint32_t)a.W) {
        static_cast<T*>(a.out)[((n * (uint32_t)a.C + c) * (uint32_t)a.H + (uint32_t)h) * (uint32_t)a.W + (uint32_t)wi] =
            acc[rh][rw];
      }
    }
}

// The block space must fit 31 bits (direct_form checks it; with padding far larger than the image it
// does not, and the one-element-per-thread kernel, whose index space is dx itself, runs instead).
template <typename T, int KH, int KW, int S>
int launch_bwd_blocks(const DirectArgs& src, hipStream_t s) {
  DirectArgs a = src;
  a.BH = (a.H + a.ph + S - 1) / S;
  a.BW = (a.W + a.pw + S - 1) / S;
  a.mBH = make_magic((uint32_t)a.BH);
  a.mBW = make_magic((uint32_t)a.BW);
  a.block_items = (uint32_t)a.N * (uint32_t)a.C * (uint32_t)a.BH * (uint32_t)a.BW;
  const dim3 grid((a.block_items + 255u) / 256u);
  hipLaunchKernelGGL((direct_bwd_blocks_kernel<T, KH, KW, S>), grid, dim3(256), 0, s, a);
  return (int)hipGetLastError();
}

// Backward data of a stride-2 "same" layer (pad = (k-1)/2 both ways, dilation 1) on rows of a
// multiple of four elements: a thread owns dx rows 2t, 2t+1 and columns 4q .. 4q+3 and stores them
// as two four-element rows.  With h + PH = 2a + rh, tap i reaches row h exactly when i has the
// parity of rh, and then reads dy row a - i/2; all of that is known at compile time per (row,
// column) of the block, so the loops below fold to the taps that apply.
template <typename T, int KH, int KW>
__global__ __launch_bounds__(256) void direct_bwd_s2_vec_kernel(const DirectArgs a) {
  constexpr int PH = (KH - 1) / 2, PW = (KW - 1) / 2;
  constexpr int DR0 = (PH >> 1) - (KH - 1) / 2, DR1 = (1 + PH) >> 1, NR = DR1 - DR0 + 1;
  constexpr int DC0 = (PW >> 1) - (KW - 1) / 2, DC1 = (3 + PW) >> 1, NC = DC1 - DC0 + 1;
  const uint32_t idx = xcd_contiguous_block_id() * 256u + threadIdx.x;
  if (idx >= a.block_items) return;
  const uint32_t q1 = mdiv(idx, a.mBW), q = idx - q1 * (uint32_t)a.BW;
  const uint32_t q2 = mdiv(q1, a.mBH), t = q1 - q2 * (uint32_t)a.BH;
  const uint32_t n = mdiv(q2, a.mC), c = q2 - n * (uint32_t)a.C;
  const uint32_t g = mdiv(c, a.mCg), cl = c - g * (uint32_t)a.Cg;
  const uint32_t P = (uint32_t)(a.OH * a.OW);
  const T* dy = static_cast<const T*>(a.in) + (n * (uint32_t)a.K + g * (uint32_t)a.Kg) * P;
  const T* w = static_cast<const T*>(a.w) + (g * (uint32_t)a.Kg * (uint32_t)a.Cg + cl) * (uint32_t)(KH * KW);
  T acc[2][4];
#pragma unroll
  for (int r = 0; r < 2; ++r)
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[r][v] = T(0);
  for (int k = 0; k < a.Kg; ++k) {
    const T* wk = w + (uint32_t)k * (uint32_t)a.Cg * (uint32_t)(KH * KW);
    const T* dk = dy + (uint32_t)k * P;
    T wv[KH][KW];
#pragma unroll
    for (int i = 0; i < KH; ++i)
#pragma unroll
      for (int j = 0; j < KW; ++j) wv[i][j] = wk[i * KW + j];
    T dv[NR][NC];
#pragma unroll
    for (int dr = 0; dr < NR; ++dr)
#pragma unroll
      for (int dc = 0; dc < NC; ++dc) {
        const int oh = (int)t + DR0 + dr, ow = 2 * (int)q + DC0 + dc;
        const bool ok = ((uint32_t)oh < (uint32_t)a.OH) & ((uint32_t)ow < (uint32_t)a.OW);
        const T val = dk[ok ? oh * a.OW + ow : 0];
        dv[dr][dc] = ok ? val : T(0);
      }
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
      for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int i = 0; i < KH; ++i)
#pragma unroll
          for (int j = 0; j < KW; ++j)
            if ((i & 1) == ((r + PH) & 1) && (j & 1) == ((v + PW) & 1))
              acc[r][v] += wv[i][j] * dv[((r + PH) >> 1) - (i >> 1) - DR0][((v + PW) >> 1) - (j >> 1) - DC0];
  }
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const uint32_t h = 2u * t + (uint32_t)r;
    if (h < (uint32_t)a.H) {
      Vec4<T>* dst = reinterpret_cast<Vec4<T>*>(static_cast<T*>(a.out) +
                                                ((n * (uint32_t)a.C + c) * (uint32_t)a.H + h) * (uint32_t)a.W + 4u * q);
      Vec4<T> o;
#pragma unroll
      for (int v = 0; v < 4; ++v) o.v[v] = acc[r][v];
      *dst = o;
    }
  }
}

template <typename T, int KH, int KW>
int launch_bwd_s2_vec(const DirectArgs& src, hipStream_t s) {
  DirectArgs a = src;
  a.BH = (a.H + 1) / 2;
  a.BW = a.W / 4;
  a.mBH = make_magic((uint32_t)a.BH);
  a.mBW = make_magic((uint32_t)a.BW);
  a.block_items = (uint32_t)a.N * (uint32_t)a.C * (uint32_t)a.BH * (uint32_t)a.BW;
  const dim3 grid((a.block_items + 255u) / 256u);
  hipLaunchKernelGGL((direct_bwd_s2_vec_kernel<T, KH, KW>), grid, dim3(256), 0, s, a);
  return (int)hipGetLastError();
}

template <typename T, int KH, int KW>
int launch_direct_k(int pass, const DirectArgs& a, hipStream_t s) {
  if (pass == 0) {
    hipLaunchKernelGGL((direct_fwd_kernel<T, KH, KW>), dim3((a.y_elems + 255u) / 256u), dim3(256), 0, s, a);
  } else {
    hipLaunchKernelGGL((direct_bwd_data_kernel<T, KH, KW>), dim3((a.x_elems + 255u) / 256u), dim3(256), 0, s, a);
  }
  return (int)hipGetLastError();
}

// The rows-per-thread kernels.  Backward data (stride 1 only) runs as the forward pass of the mirrored
// problem: dy is the input blob with K channels, dx the output with C channels.
template <typename T, int KH, int KW, bool UNIT>
int launch_rows(int pass, const DirectArgs& src, bool vec, hipStream_t s) {
  constexpr int kRows = rows_per_thread(UNIT);
  DirectArgs a = src;
  vec = vec && UNIT;  // the four-columns-per-thread kernels exist at unit stride and dilation only
  if (vec) {
    a.OWQ = src.W / kVecCols;
    a.mOWQ = make_magic((uint32_t)a.OWQ);
  }
  if (pass == 2 && vec) {
    a.OHB = (a.OH + kVecRows - 1) / kVecRows;
    a.mOHB = make_magic((uint32_t)a.OHB);
    hipLaunchKernelGGL((direct_wgrad_rows_vec_kernel<T, KH, KW>), dim3((uint32_t)(a.K * a.Cg), (uint32_t)a.S),
                       dim3(256), 0, s, a);
    return (int)hipGetLastError();
  }
  if (pass == 2) {
    a.OHB = (a.OH + kRows - 1) / kRows;
    a.mOHB = make_magic((uint32_t)a.OHB);
    hipLaunchKernelGGL((direct_wgrad_rows_kernel<T, KH, KW, UNIT>), dim3((uint32_t)(a.K * a.Cg), (uint32_t)a.S),
                       dim3(256), 0, s, a);
    return (int)hipGetLastError();
  }
  if (pass == 0) {
    a.w_out_stride = (uint32_t)(a.Cg * KH * KW);
    a.w_in_stride = (uint32_t)(KH * KW);
  } else {
    a.C = src.K;
    a.K = src.C;
    a.Cg = src.Kg;
    a.Kg = src.Cg;
    a.H = src.OH;
    a.W = src.OW;
    a.OH = src.H;
    a.OW = src.W;
    a.ph = src.dh * (KH - 1) - src.ph;
    a.pw = src.dw * (KW - 1) - src.pw;
    a.w_out_stride = (uint32_t)(KH * KW);
    a.w_in_stride = (uint32_t)(src.Cg * KH * KW);
    a.mOW = src.mW;
    a.mK = src.mC;
    a.mKg = src.mCg;
  }
  if (vec) {
    a.OHB = (a.OH + kVecRows - 1) / kVecRows;
    a.mOHB = make_magic((uint32_t)a.OHB);
    a.row_items = (uint32_t)a.N * (uint32_t)a.K * (uint32_t)a.OHB * (uint32_t)a.OWQ;
    const dim3 vgrid((a.row_items + 255u) / 256u);
    if (pass == 0)
      hipLaunchKernelGGL((direct_rows_vec_kernel<T, KH, KW, false>), vgrid, dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL((direct_rows_vec_kernel<T, KH, KW, true>), vgrid, dim3(256), 0, s, a);
    return (int)hipGetLastError();
  }
  a.OHB = (a.OH + kRows - 1) / kRows;
  a.mOHB = make_magic((uint32_t)a.OHB);
  a.row_items = (uint32_t)a.N * (uint32_t)a.K * (uint32_t)a.OHB * (uint32_t)a.OW;
  const dim3 grid((a.row_items + 255u) / 256u);
  if (pass == 0)
    hipLaunchKernelGGL((direct_rows_kernel<T, KH, KW, UNIT, false>), grid, dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL((direct_rows_kernel<T, KH, KW, UNIT, true>), grid, dim3(256), 0, s, a);
  return (int)hipGetLastError();
}

template <typename T>
int launch_direct_t(int pass, const DirectArgs& a, hipStream_t s) {
  const DirectForm f = direct_form(pass, a, sizeof(T));
  const bool k3 = a.kh == 3;
  switch (f.kind) {
    case DF_S2: return k3 ? launch_s2<T, 3, 3>(pass, a, s) : launch_s2<T, 5, 5>(pass, a, s);
    case DF_ROWS:
    case DF_ROWS_VEC: {
      const bool vec = f.kind == DF_ROWS_VEC;
      if (k3) return f.unit ? launch_rows<T, 3, 3, true>(pass, a, vec, s) : launch_rows<T, 3, 3, false>(pass, a, vec, s);
      return f.unit ? launch_rows<T, 5, 5, true>(pass, a, vec, s) : launch_rows<T, 5, 5, false>(pass, a, vec, s);
    }
    case DF_WGRAD_TAPS:
      hipLaunchKernelGGL(direct_wgrad_kernel<T>, dim3((uint32_t)(a.K * a.Cg), (uint32_t)a.S), dim3(256), 0, s, a);
      return (int)hipGetLastError();
    case DF_BWD_S2_VEC: return k3 ? launch_bwd_s2_vec<T, 3, 3>(a, s) : launch_bwd_s2_vec<T, 5, 5>(a, s);
    case DF_BWD_BLOCKS: return k3 ? launch_bwd_blocks<T, 3, 3, 2>(a, s) : launch_bwd_blocks<T, 5, 5, 2>(a, s);
    case DF_ELEM_K3: return launch_direct_k<T, 3, 3>(pass, a, s);
    default: return launch_direct_k<T, 0, 0>(pass, a, s);
  }
}

}  // namespace

// Which kernel a pass of a thin-group descriptor runs.  The choice depends on the layer parameters and
// on the alignment of the blobs of the call (the 16-byte forms need aligned rows); null pointers
// stand for fully aligned blobs, which is what the descriptor's kernel names assume.
DirectForm direct_form(int pass, const DirectArgs& a, size_t elem) {
  DirectForm f = {DF_ELEM, false};
  const bool k3 = a.kh == 3 && a.kw == 3, k5 = a.kh == 5 && a.kw == 5;
  const int KH = a.kh, KW = a.kw;
  const uintptr_t in = (uintptr_t)a.in, out = (uintptr_t)a.out, w = (uintptr_t)a.w;
  const uintptr_t m4 = 4 * elem - 1, m2 = 2 * elem - 1;
  f.unit = a.sh == 1 && a.sw == 1 && a.dh == 1 && a.dw == 1;
  const bool s2d1 = a.sh == 2 && a.sw == 2 && a.dh == 1 && a.dw == 1;
  if (pass != 1 && (k3 || k5)) {
    // stride 2 with "same" padding along rows of a multiple of four elements: x by 16-byte accesses,
    // y (forward) or dy (filter gradient) by two-element ones
    const uintptr_t other = pass == 0 ? out : w;
    if (s2d1 && a.W % 4 == 0 && a.pw == (KW - 1) / 2 && 2 * a.OW == a.W && (in & m4) == 0 && (other & m2) == 0) {
      f.kind = DF_S2;
      return f;
    }
  }
  const bool rows_ok = pass != 1 || (a.sh == 1 && a.sw == 1);  // backward data: stride 1 only
  if (rows_ok && (k3 || k5)) {
    // four columns per thread: unit stride and dilation, "same" padding along the row, rows of a
    // multiple of four elements, every blob of the pass 16-byte aligned for its base type
    const bool aligned = ((in | out | (pass == 2 ? w : 0)) & m4) == 0;
    const bool vec = f.unit && aligned && a.W % 4 == 0 && a.pw == (KW - 1) / 2 && a.OW == a.W;
    f.kind = vec ? DF_ROWS_VEC : DF_ROWS;
    return f;
  }
  if (pass == 2) {
    f.kind = DF_WGRAD_TAPS;
    return f;
  }
  if (pass == 1 && s2d1 && (k3 || k5)) {
    if (a.W % 4 == 0 && a.ph == (KH - 1) / 2 && a.pw == (KW - 1) / 2 && (out & m4) == 0) {
      f.kind = DF_BWD_S2_VEC;
      return f;
    }
    const unsigned long long items = (unsigned long long)a.N * (unsigned long long)a.C *
                                     (unsigned long long)((a.H + a.ph + 1) / 2) *
                                     (unsigned long long)((a.W + a.pw + 1) / 2);
    if (items < (1ull << 31)) {
      f.kind = DF_BWD_BLOCKS;
      return f;
    }
  }
  f.kind = k3 ? DF_ELEM_K3 : DF_ELEM;
  return f;
}

void direct_form_name(int pass, const DirectArgs& a, char* buf, size_t len) {
  const DirectForm f = direct_form(pass, a, 4);
  static const char* kinds[] = {"elem", "elem_k3", "rows", "rows_vec", "s2", "bwd_s2_vec", "bwd_blocks", "wgrad_taps"};
  const bool sized = f.kind != DF_ELEM && f.kind != DF_ELEM_K3 && f.kind != DF_WGRAD_TAPS;
  if (sized)
    snprintf(buf, len, "%s_k%d%s", kinds[f.kind], a.kh, (f.kind == DF_ROWS && f.unit) ? "_unit" : "");
  else
    snprintf(buf, len, "%s", kinds[f.kind]);
}

int launch_direct(int pass, const DirectArgs& a, bool f64, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  return f64 ? launch_direct_t<double>(pass, a, s) : launch_direct_t<float>(pass, a, s);
}

}  // namespace mi355conv
