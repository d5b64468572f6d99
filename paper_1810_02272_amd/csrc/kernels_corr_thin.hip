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

// ---- the same GEMM with the gathered rows staged in LDS -------------------------------------
// For stride-1, dilation-1 gathers with 3x3 or 5x5 taps (every first-layer backward-data pass of
// such a layer) the form above is bound by one cache access per column and k row.  Here
// a workgroup covers 128 columns, two per lane (col and col + 64), and first brings the raw input
// rows those columns touch into LDS -- a zero-padded patch as in corr_patch_kernel, all channels of
// the group at once -- with loads that write LDS themselves: lane l of a wave fills word l of a
// 64-word segment, a word outside the image presents an offset beyond the blob and receives the zero
// the range check returns, lanes past the channel's patch are switched off.  Wave w loads and
// multiplies the channels w, w + 4, ...; a tap is then an LDS read at the column's patch position
// plus an immediate offset, and the four waves' sums are added through LDS in wave order.
// The A operands are scalar loads from the weight blob itself (no pack kernel): row m, gathered
// channel c, tap t sit at w_grp_stride*g + w_row_stride*m + w_chan_stride*c + t, with the taps
// running backwards in the backward-data pass (REV).
constexpr int kTlCols = 128;      // columns per workgroup
constexpr int kTlMaxSeg = 8;      // 64-word segments of a channel's patch: PSZ <= 512 floats

typedef __attribute__((address_space(3))) void* ThinLdsPtr;
typedef __attribute__((address_space(4))) float ConstFloat;

template <int ROWS, int TW, bool REV>
__global__ __launch_bounds__(256) void corr_thin_lds_kernel(const CorrArgs a) {
  extern __shared__ __align__(16) float lds[];  // [Cg_in][PSZ] patch; afterwards [4][ROWS][kTlCols] sums
  const int t = threadIdx.x, lane = t & 63;
  const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
  const uint32_t col_tile = blockIdx.x % (uint32_t)a.col_tiles;
  const uint32_t g = blockIdx.x / (uint32_t)a.col_tiles;

  // geometry of this tile's patch (uniform), as in corr_patch_kernel: the columns run through one or
  // more images; segment 0 starts at output row a0 of image n0 and owns patch rows 0 .. R0-1, every
  // later segment starts at output row 0 and owns RS = PH + TH - 1 patch rows
  constexpr int TH = TW, T = TW * TW;  // square kernels only
  const uint32_t col0 = col_tile * kTlCols;
  const uint32_t n0 = mdiv(col0, a.mP);
  const uint32_t a0 = mdiv(col0 - n0 * a.P, a.mPW);
  const uint32_t R0 = (uint32_t)a.PH - a0 + TH - 1;
  const uint32_t RS = (uint32_t)a.PH + TH - 1;
  auto patch_row_base = [&](uint32_t n, uint32_t pa) {
    const uint32_t s = n - n0;
    return s == 0 ? pa - a0 : R0 + (s - 1) * RS + pa;
  };
  uint32_t col_last = col0 + kTlCols - 1;
  if (col_last > (uint32_t)a.ncols - 1) col_last = (uint32_t)a.ncols - 1;
  uint32_t patch_elems;
  {
    const uint32_t n = mdiv(col_last, a.mP);
    const uint32_t pa = mdiv(col_last - n * a.P, a.mPW);
    patch_elems = (patch_row_base(n, pa) + TH) * (uint32_t)a.PWID;
  }

  // this lane's two columns: patch position under tap (0, 0) and place in the output ("not stored" =
  // beyond the blob); a column past the edge computes on the last real column and stores nothing
  uint32_t cb[2], coff[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const uint32_t col = col0 + (uint32_t)lane + 64u * j;
    const uint32_t colc = col > col_last ? col_last : col;
    const uint32_t n = mdiv(colc, a.mP);
    const uint32_t pix = colc - n * a.P;
    const uint32_t pa = mdiv(pix, a.mPW);
    const uint32_t pb = pix - pa * a.PW;
    cb[j] = patch_row_base(n, pa) * (uint32_t)a.PWID + pb;
    const int hh = (int)pa * a.OSh - a.opad_h, ww = (int)pb * a.OSw - a.opad_w;
    coff[j] = 0x40000000u;
    if (col <= col_last && (uint32_t)hh < (uint32_t)a.OHd && (uint32_t)ww < (uint32_t)a.OWd)
      coff[j] = 4u * (n * (uint32_t)a.out_img_stride + (uint32_t)hh * (uint32_t)a.OWd + (uint32_t)ww);
  }

  // where the patch words this lane fills come from (channel 0 of the group): word 64*s + lane
  const __amdgpu_buffer_rsrc_t in_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.in), 0, (int)a.in_bytes, 0x00020000);
  const int nfull = a.PSZ / 64;          // segments that lie inside a channel's patch with all 64 words
  const int tail = a.PSZ - 64 * nfull;   // words of the segment after them (PSZ <= 64 * kTlMaxSeg)
  uint32_t psrc[kTlMaxSeg];
#pragma unroll
  for (int s = 0; s < kTlMaxSeg; ++s) {
    const uint32_t e = (uint32_t)(64 * s + lane);
    uint32_t src = 0x80000000u;
    if (64 * s < a.PSZ && e < patch_elems) {
      const uint32_t prow = mdiv(e, a.mPWID);
      const uint32_t pcol = e - prow * a.PWID;
      uint32_t n = n0, rin = prow, alo = a0;
      if (prow >= R0) {
        const uint32_t s1 = mdiv(prow - R0, a.mRSEG);
        n = n0 + 1 + s1;
        rin = prow - R0 - s1 * RS;
        alo = 0;
      }
      const int ih = (int)(alo + rin) - a.ph, iw = (int)pcol - a.pw;
      if ((uint32_t)ih < (uint32_t)a.IH && (uint32_t)iw < (uint32_t)a.IW && n < (uint32_t)a.Nimg)
        src = 4u * (n * (uint32_t)a.in_img_stride + g * (uint32_t)a.in_grp_stride + (uint32_t)ih * a.IW + iw);
    }
    psrc[s] = src;
  }
  // all of this wave's channels in flight at once; an offset of 2^31 plus a channel displacement of at
  // most 2^30 stays beyond the blob
  const uint32_t chan_bytes = 4u * (uint32_t)a.IHW;
  for (int c = wv; c < a.Cg_in; c += 4) {
    const uint32_t cdisp = (uint32_t)c * chan_bytes;
#pragma unroll
    for (int s = 0; s < kTlMaxSeg; ++s) {
      if (s < nfull)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(in_rsrc, (ThinLdsPtr)(lds + c * a.PSZ + 64 * s), 4, psrc[s] + cdisp, 0,
                                                 0, 0);
      else if (s == nfull && lane < tail)  // the words past it belong to the next channel
        __builtin_amdgcn_raw_ptr_buffer_load_lds(in_rsrc, (ThinLdsPtr)(lds + c * a.PSZ + 64 * s), 4, psrc[s] + cdisp, 0,
                                                 0, 0);
    }
  }

  float acc[2][ROWS];
#pragma unroll
  for (int m = 0; m < ROWS; ++m) acc[0][m] = acc[1][m] = 0.f;
  // uniform addresses into a blob that is read-only for the whole kernel: the constant address space
  // makes these scalar loads
  const ConstFloat* wg = (const ConstFloat*)(a.A + (size_t)g * a.w_grp_stride);
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's words are in LDS
  __syncthreads();
  for (int c = wv; c < a.Cg_in; c += 4) {
    const float* x0 = lds + c * a.PSZ + cb[0];
    const float* x1 = lds + c * a.PSZ + cb[1];
    const ConstFloat* wk = wg + (size_t)c * a.w_chan_stride;
#pragma unroll
    for (int ti = 0; ti < TH; ++ti) {
      float xa[TW], xb[TW];
#pragma unroll
      for (int tj = 0; tj < TW; ++tj) {
        xa[tj] = x0[ti * a.PWID + tj];
        xb[tj] = x1[ti * a.PWID + tj];
      }
#pragma unroll
      for (int m = 0; m < ROWS; ++m)
#pragma unroll
        for (int tj = 0; tj < TW; ++tj) {
          const int tap = ti * TW + tj;
          const float av = wk[(size_t)m * a.w_row_stride + (REV ? T - 1 - tap : tap)];
          acc[0][m] += av * xa[tj];
          acc[1][m] += av * xb[tj];
        }
    }
  }

  __syncthreads();     // every wave is done with the patch: the sums take its place
  float* red = lds;    // [4][ROWS][kTlCols]
#pragma unroll
  for (int m = 0; m < ROWS; ++m) {
    red[(wv * ROWS + m) * kTlCols + lane] = acc[0][m];
    red[(wv * ROWS + m) * kTlCols + 64 + lane] = acc[1][m];
  }
  __syncthreads();
  if (wv > 1) return;  // wave 0 stores the columns lane, wave 1 the columns lane + 64

  const uint32_t my_coff = wv == 0 ? coff[0] : coff[1];
  const __amdgpu_buffer_rsrc_t out_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(a.out, 0, (int)(4u * (uint32_t)a.out_elems), 0x00020000);
#pragma unroll
  for (int m = 0; m < ROWS; ++m) {
    if (m >= a.Mrows) break;
    const uint32_t chan = g * (uint32_t)a.chan_per_grp + (uint32_t)m;
    const uint32_t off = 4u * chan * (uint32_t)(a.OHd * a.OWd) + my_coff;
    const float* r = red + m * kTlCols + 64 * wv + lane;
    float v = ((r[0] + r[ROWS * kTlCols]) + r[2 * ROWS * kTlCols]) + r[3 * ROWS * kTlCols];
    if (a.bias) v += a.bias[chan];
    if (a.accumulate) v += __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(out_rsrc, off, 0, 0));
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), out_rsrc, off, 0, 0);
  }
}

// LDS of a workgroup: the patch, or the four waves' sums where those need more
inline size_t thin_lds_bytes(const CorrArgs& a) {
  const size_t patch = (size_t)a.Cg_in * a.PSZ, sums = (size_t)4 * 4 * kTlCols;
  return (patch > sums ? patch : sums) * sizeof(float);
}

template <int ROWS, int TW>
int launch_thin_lds_rt(CorrArgs a, hipStream_t s) {
  a.col_tiles = (a.ncols + kTlCols - 1) / kTlCols;
  const dim3 grid((uint32_t)a.G * (uint32_t)a.col_tiles), block(256);
  const size_t lds = thin_lds_bytes(a);
  if (a.w_reversed)
    hipLaunchKernelGGL((corr_thin_lds_kernel<ROWS, TW, true>), grid, block, lds, s, a);
  else
    hipLaunchKernelGGL((corr_thin_lds_kernel<ROWS, TW, false>), grid, block, lds, s, a);
  return (int)hipGetLastError();
}

template <int ROWS>
int launch_thin_lds_r(const CorrArgs& a, hipStream_t s) {
  return a.TW == 3 ? launch_thin_lds_rt<ROWS, 3>(a, s) : launch_thin_lds_rt<ROWS, 5>(a, s);
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

// The caller guarantees: 1 <= Mrows <= 4, the offset-only epilogue applies, no split of the reduction;
// use_patch selects the LDS-staged form (the patch and w_* fields are then set and A is the weight blob).
int launch_corr_thin(const CorrArgs& a, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  if (a.Mrows < 1 || a.Mrows > 4 || !a.simple_epilogue || a.ksplit > 1 || a.ncols < 1) return (int)hipErrorInvalidValue;
  if (a.use_patch) {
    if ((a.TW != 3 && a.TW != 5) || a.THW != a.TW * a.TW || a.PSZ < 1 || a.PSZ > 64 * kTlMaxSeg || a.Cg_in < 1 ||
        thin_lds_bytes(a) > 64 * 1024 || a.in_bytes > (1u << 30))
      return (int)hipErrorInvalidValue;
    switch (a.Mrows) {
      case 1: return launch_thin_lds_r<1>(a, s);
      case 2: return launch_thin_lds_r<2>(a, s);
      case 3: return launch_thin_lds_r<3>(a, s);
      default: return launch_thin_lds_r<4>(a, s);
    }
  }
  switch (a.Mrows) {
    case 1: return launch_thin_r<1>(a, s);
    case 2: return launch_thin_r<2>(a, s);
    case 3: return launch_thin_r<3>(a, s);
    default: return launch_thin_r<4>(a, s);
  }
}

}  // namespace mi355conv
