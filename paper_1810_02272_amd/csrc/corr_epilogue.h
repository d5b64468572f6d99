// Epilogue shared by the correlation kernels: bias add and scatter of the accumulator tile.
#pragma once

#include <hip/hip_runtime.h>

#include "device_utils.h"
#include "internal.h"

namespace mi355conv {

// Two LDS tables turn an accumulator into its output address with one 16-byte read per row:
//   rowtab[m]   = {offset, row shift, column shift, bias}   (row m = (channel, row phase, column phase))
//   coltab[col] = {offset, row, column, -}                   (column = (image, a, b))
// An element is stored when (row shift + row, column shift + column) lies inside the output
// image; rows past the matrix edge and columns past the batch carry a shift that fails the test.
// Must be entered after a barrier: the tables overwrite the pipeline buffers at `smem`.
template <int MT, int MB, int NB, int BM, int BN, typename Acc>
__device__ __forceinline__ void corr_epilogue(const CorrArgs& a, float* smem, Acc (&acc)[MB][NB], uint32_t m_tile,
                                              uint32_t col_tile, uint32_t g, int wm, int wn, uint32_t split = 0) {
  using M = Mfma<MT>;
  // With a split reduction every split writes its raw partial sums, in the output blob's own
  // layout, to its slice of the workspace; a reduce kernel adds the slices and the bias.
  float* const out = a.ksplit > 1 ? a.part + (size_t)split * a.out_elems : a.out;
  const float* const bias = a.ksplit > 1 ? nullptr : a.bias;
  const bool accumulate = a.accumulate != 0 && a.ksplit <= 1;
  const int t = threadIdx.x, lane = t & 63;
  int4* rowtab = reinterpret_cast<int4*>(smem);
  int4* coltab = rowtab + BM;
  if (a.simple_epilogue) {
    // One output phase per channel (forward, stride-1 backward data, InnerProduct) and an output blob
    // of at most 2^30 bytes: whether an element is stored depends on its row and on its column
    // separately, so the tables hold byte offsets with an out-of-range value for "not stored"
    // (2^31 for a row, 2^30 for a column: any sum with one of them lies beyond the blob) and the
    // range check of the buffer store drops those elements -- one add per element, no compares.
    for (int m = t; m < BM; m += 256) {
      const uint32_t gm = m_tile * BM + m;
      uint32_t off = 0x80000000u;
      float bb = 0.f;
      if (gm < (uint32_t)a.Mrows) {
        const uint32_t chan = g * a.chan_per_grp + gm;
        off = 4u * chan * (uint32_t)(a.OHd * a.OWd);
        if (bias) bb = bias[chan];
      }
      rowtab[m] = make_int4((int)off, 0, 0, __builtin_bit_cast(int, bb));
    }
    for (int cl = t; cl < BN; cl += 256) {
      const uint32_t col = col_tile * BN + cl;
      uint32_t off = 0x40000000u;
      if (col < (uint32_t)a.ncols) {
        const uint32_t n = mdiv(col, a.mP);
        const uint32_t pix = col - n * a.P;
        const uint32_t pa = mdiv(pix, a.mPW);
        const uint32_t pb = pix - pa * a.PW;
        const int hh = (int)pa * a.OSh - a.opad_h, ww = (int)pb * a.OSw - a.opad_w;
        if ((uint32_t)hh < (uint32_t)a.OHd && (uint32_t)ww < (uint32_t)a.OWd)
          off = 4u * (n * (uint32_t)a.out_img_stride + (uint32_t)hh * (uint32_t)a.OWd + (uint32_t)ww);
      }
      coltab[cl] = make_int4((int)off, 0, 0, 0);
    }
    __syncthreads();
    const __amdgpu_buffer_rsrc_t out_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(out, 0, (int)(4u * (uint32_t)a.out_elems), 0x00020000);
    uint32_t co[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) co[j] = (uint32_t)coltab[(wn * NB + j) * MT + lane % MT].x;
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int r = 0; r < M::NR; ++r) {
        const int4 rt = rowtab[(wm * MB + i) * MT + M::row(r, lane)];
        const float bb = __builtin_bit_cast(float, rt.w);
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          const uint32_t off = (uint32_t)rt.x + co[j];
          float v = acc[i][j][r] + bb;
          if (accumulate) v += __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(out_rsrc, off, 0, 0));
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), out_rsrc, off, 0, 0);
        }
      }
    return;
  }
  for (int m = t; m < BM; m += 256) {
    const uint32_t gm = m_tile * BM + m;
    int off = 0, hh = -(1 << 28), ww = 0;
    float bb = 0.f;
    if (gm < (uint32_t)a.Mrows) {
      const uint32_t c = mdiv(gm, a.mRShw);
      const uint32_t rem = gm - c * a.RShw;
      uint32_t rh = mdiv(rem, a.mRSw);
      uint32_t rw = rem - rh * a.RSw;
      if (a.tab_h) rh = (uint32_t)a.phase_h[rh];
      if (a.tab_w) rw = (uint32_t)a.phase_w[rw];
      const uint32_t chan = g * a.chan_per_grp + c;
      hh = (int)rh - a.opad_h;
      ww = (int)rw - a.opad_w;
      off = (int)(chan * (uint32_t)(a.OHd * a.OWd)) + hh * a.OWd + ww;
      if (bias) bb = bias[chan];
    }
    rowtab[m] = make_int4(off, hh, ww, __builtin_bit_cast(int, bb));
  }
  for (int cl = t; cl < BN; cl += 256) {
    const uint32_t col = col_tile * BN + cl;
    int off = 0, hh = -(1 << 28), ww = 0;
    if (col < (uint32_t)a.ncols) {
      const uint32_t n = mdiv(col, a.mP);
      const uint32_t pix = col - n * a.P;
      const uint32_t pa = mdiv(pix, a.mPW);
      const uint32_t pb = pix - pa * a.PW;
      hh = (int)pa * a.OSh;
      ww = (int)pb * a.OSw;
      off = (int)(n * (uint32_t)a.out_img_stride) + hh * a.OWd + ww;
    }
    coltab[cl] = make_int4(off, hh, ww, 0);
  }
  __syncthreads();

  int4 ct[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) ct[j] = coltab[(wn * NB + j) * MT + lane % MT];
  if ((uint32_t)a.out_elems < (1u << 29)) {
    // Output below 2^31 bytes: an element that is not stored gets the offset 2^31 and the range check
    // of the buffer store drops it -- no branch around the store, 32-bit offsets.
    const __amdgpu_buffer_rsrc_t out_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(out, 0, (int)(4u * (uint32_t)a.out_elems), 0x00020000);
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int r = 0; r < M::NR; ++r) {
        const int4 rt = rowtab[(wm * MB + i) * MT + M::row(r, lane)];
        const float bb = __builtin_bit_cast(float, rt.w);
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          const int hh = rt.y + ct[j].y, ww = rt.z + ct[j].z;
          const bool ok = ((uint32_t)hh < (uint32_t)a.OHd) & ((uint32_t)ww < (uint32_t)a.OWd);
          const uint32_t off = ok ? 4u * (uint32_t)(rt.x + ct[j].x) : 0x80000000u;
          float v = acc[i][j][r] + bb;
          if (accumulate) v += __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(out_rsrc, off, 0, 0));
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), out_rsrc, off, 0, 0);
        }
      }
    return;
  }
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int r = 0; r < M::NR; ++r) {
      const int4 rt = rowtab[(wm * MB + i) * MT + M::row(r, lane)];
      const float bb = __builtin_bit_cast(float, rt.w);
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int hh = rt.y + ct[j].y, ww = rt.z + ct[j].z;
        if ((uint32_t)hh < (uint32_t)a.OHd && (uint32_t)ww < (uint32_t)a.OWd) {
          float* const dst = out + (rt.x + ct[j].x);
          const float v = acc[i][j][r] + bb;
          *dst = accumulate ? *dst + v : v;
        }
      }
    }
}

}  // namespace mi355conv
