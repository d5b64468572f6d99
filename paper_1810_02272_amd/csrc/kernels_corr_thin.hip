// Correlation kernel for gfx950 for GEMMs of at most four rows per group:
//   D[m][col] = sum_k A[m][k] * gather(in)[k][col],  m < ROWS <= 4
// -- the backward-data pass of a layer with one to four input channels per group at stride 1 (the
// first layer of a network: one or three image planes), or a forward pass with that few outputs.  The
// matrix tiles of corr_kernel start at 16 rows, so such a GEMM wastes three quarters or more of
// every matrix instruction there; here each lane owns one column and keeps ROWS sums, the
// products are plain fused multiply-adds whose A operand is a scalar register, and the k-table
// entries and the packed A rows (both uniform over a wave) arrive through scalar loads.
//
// A workgroup covers 64 columns; its four waves take the k rows in groups of eight in turn (wave w
// the groups w, w + 4, ...) and their partial sums are added through LDS in wave order, so the
// result does not depend on scheduling.  The gather, its three bounds modes and the k table are those of
// corr_kernel; the epilogue is the offset-only form (one output phase per channel, output blob of
// at most 2^30 bytes), which is the only case the host code selects this kernel for.
#include <hip/hip_runtime.h>

#include "device_utils.h"
#include "internal.h"

namespace mi355conv {

namespace {

constexpr int kThinCols = 64;  // columns per workgroup
constexpr int kThinK = 8;      // k rows fetched together

template <int ROWS, int MODE>
__global__ __launch_bounds__(256) void corr_thin_kernel(const CorrArgs a) {
  __shared__ float red[4][ROWS][kThinCols];
  const int t = threadIdx.x, lane = t & 63;
  const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
  const uint32_t col_tile = blockIdx.x % (uint32_t)a.col_tiles;
  const uint32_t g = blockIdx.x / (uint32_t)a.col_tiles;

  // column state of the gather, as in corr_kernel: an element that must read as zero gets an
  // offset at or beyond the buffer size
  const uint32_t col = col_tile * kThinCols + lane;
  uint32_t cbase = MODE == 0 ? 0x80000000u : 0u, cinv = 0;
  int cih0 = -(1 << 29), ciw0 = 0;
  if (col < (uint32_t)a.ncols) {
    const uint32_t n = mdiv(col, a.mP);
    const uint32_t pix = col - n * a.P;
    const uint32_t pa = mdiv(pix, a.mPW);
    const uint32_t pb = pix - pa * a.PW;
    cih0 = (int)pa * a.sh - a.ph;
    ciw0 = (int)pb * a.sw - a.pw;
    cbase = 4u * (uint32_t)((int)(n * a.in_img_stride + g * a.in_grp_stride) + cih0 * a.IW + ciw0);
  }
  if (MODE == 2) {  // bit `tap` set: that tap of this column lies outside the image
    const int TH = a.THW / a.TW;
    for (int i = 0, tap = 0; i < TH; ++i)
      for (int j = 0; j < a.TW; ++j, ++tap) {
        const bool ok = ((uint32_t)(cih0 + i * a.dh) < (uint32_t)a.IH) & ((uint32_t)(ciw0 + j * a.dw) < (uint32_t)a.IW);
        cinv |= ok ? 0u : (1u << tap);
      }
  }
  const __amdgpu_buffer_rsrc_t in_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.in), 0, (int)a.in_bytes, 0x00020000);
  const float* Ag = a.A + (size_t)g * a.MP * a.KP;

  float acc[ROWS];
#pragma unroll
  for (int m = 0; m < ROWS; ++m) acc[m] = 0.f;

  // Groups of kThinK k rows; wave w takes the groups w, w + 4, ...  The gathered values of kRing groups
  // are in flight per wave: a ring of register sets, each refilled as soon as it has been multiplied
  // (two to four sets measure alike, six lose: the kernel is bound by the gather's cache accesses,
  // one per column and k row, as the matrix-unit kernels are on these shapes).  Everything the loop
  // does is unconditional -- a refill past the wave's last group repeats that group into a set
  // nobody multiplies -- so the sets stay in fixed registers, and the k-table entries and A operands
  // (uniform over the wave) come through scalar loads off two running pointers.
  const int ngroups = a.KP / kThinK;             // KP is a multiple of 16
  const int n_my = (ngroups - wv + 3) / 4;       // groups of this wave
  constexpr int kRing = 3;
  constexpr int kStep = 4 * kThinK;              // k rows between two groups of a wave
  float xv[kRing][kThinK];
  const KTabEntry* tp = a.ktab + wv * kThinK;    // the group gathered next
  const KTabEntry* const tlast = a.ktab + (wv + 4 * (n_my - 1)) * kThinK;
  const float* ap = Ag + wv * kThinK;            // the group multiplied next (row m at ap + m*KP)
  auto gather = [&](float(&x)[kThinK]) {
#pragma unroll
    for (int e = 0; e < kThinK; ++e) {
      const KTabEntry te = tp[e];
      uint32_t off = cbase + te.koff;
      if (MODE == 1) {
        const int ih = cih0 + te.idh, iw = ciw0 + te.jdw;
        const bool ok = ((uint32_t)ih < (uint32_t)a.IH) & ((uint32_t)iw < (uint32_t)a.IW);
        off = ok ? off : a.in_bytes;
      } else if (MODE == 2) {
        off += __builtin_amdgcn_ubfe(cinv, (uint32_t)te.tap, 1u) << 31;
      }
      x[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(in_rsrc, off, 0, 0));
    }
    tp = tp + kStep <= tlast ? tp + kStep : tlast;
  };
  auto multiply = [&](const float(&x)[kThinK]) {
#pragma unroll
    for (int m = 0; m < ROWS; ++m)
#pragma unroll
      for (int e = 0; e < kThinK; ++e) acc[m] += ap[(size_t)m * a.KP + e] * x[e];
    ap += kStep;
  };
  if (n_my > 0) {
#pragma unroll
    for (int b = 0; b < kRing; ++b) gather(xv[b]);
    int i = 0;
    for (; i + kRing <= n_my; i += kRing) {
#pragma unroll
      for (int b = 0; b < kRing; ++b) {
        multiply(xv[b]);
        gather(xv[b]);
      }
    }
#pragma unroll
    for (int b = 0; b < kRing - 1; ++b)
      if (i + b < n_my) multiply(xv[b]);
  }

#pragma unroll
  for (int m = 0; m < ROWS; ++m) red[wv][m][lane] = acc[m];
  __syncthreads();
  if (wv != 0) return;

  // offset-only epilogue: byte offsets per row and per column, "not stored" = beyond the blob
  uint32_t coff = 0x40000000u;
  if (col < (uint32_t)a.ncols) {
    const uint32_t n = mdiv(col, a.mP);
    const uint32_t pix = col - n * a.P;
    const uint32_t pa = mdiv(pix, a.mPW);
    const uint32_t pb = pix - pa * a.PW;
    const int hh = (int)pa * a.OSh - a.opad_h, ww = (int)pb * a.OSw - a.opad_w;
    if ((uint32_t)hh < (uint32_t)a.OHd && (uint32_t)ww < (uint32_t)a.OWd)
      coff = 4u * (n * (uint32_t)a.out_img_stride + (uint32_t)hh * (uint32_t)a.OWd + (uint32_t)ww);
  }
  const __amdgpu_buffer_rsrc_t out_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(a.out, 0, (int)(4u * (uint32_t)a.out_elems), 0x00020000);
#pragma unroll
  for (int m = 0; m < ROWS; ++m) {
    if (m >= a.Mrows) break;
    const uint32_t chan = g * (uint32_t)a.chan_per_grp + (uint32_t)m;
    const uint32_t off = 4u * chan * (uint32_t)(a.OHd * a.OWd) + coff;
    float v = ((red[0][m][lane] + red[1][m][lane]) + red[2][m][lane]) + red[3][m][lane];
    if (a.bias) v += a.bias[chan];
    if (a.accumulate) v += __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(out_rsrc, off, 0, 0));
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), out_rsrc, off, 0, 0);
  }
}

template <int ROWS>
int launch_thin_r(CorrArgs a, hipStream_t s) {
  a.col_tiles = (a.ncols + kThinCols - 1) / kThinCols;
  const dim3 grid((uint32_t)a.G * (uint32_t)a.col_tiles), block(256);
  if (a.bounds_mode == 0)
    hipLaunchKernelGGL((corr_thin_kernel<ROWS, 0>), grid, block, 0, s, a);
  else if (a.bounds_mode == 2)
    hipLaunchKernelGGL((corr_thin_kernel<ROWS, 2>), grid, block, 0, s, a);
  else
    hipLaunchKernelGGL((corr_thin_kernel<ROWS, 1>), grid, block, 0, s, a);
  return (int)hipGetLastError();
}

}  // namespace

// The caller guarantees: 1 <= Mrows <= 4, the offset-only epilogue applies, no split of the reduction.
int launch_corr_thin(const CorrArgs& a, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  if (a.Mrows < 1 || a.Mrows > 4 || !a.simple_epilogue || a.ksplit > 1 || a.ncols < 1) return (int)hipErrorInvalidValue;
  switch (a.Mrows) {
    case 1: return launch_thin_r<1>(a, s);
    case 2: return launch_thin_r<2>(a, s);
    case 3: return launch_thin_r<3>(a, s);
    default: return launch_thin_r<4>(a, s);
  }
}

}  // namespace mi355conv
