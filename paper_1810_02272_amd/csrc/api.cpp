// Host side of the C boundary: parameter validation, shape arithmetic, kernel-variant choice,
// workspace sizing and the five entry points.  No device memory is allocated anywhere here, and
// conv_desc_create touches no device at all (it also runs on machines without a GPU).
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "internal.h"

using namespace mi355conv;

namespace {

thread_local int g_last_hip_error = 0;

constexpr int64_t kMaxElems = (int64_t)1 << 30;  // 32-bit byte offsets in the kernels

int64_t floor_div(int64_t a, int64_t b) {
  int64_t q = a / b;
  if ((a % b) != 0 && ((a < 0) != (b < 0))) --q;
  return q;
}

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

// Row tile: the smallest padded row count wins; a taller tile is taken over a shorter one when it
// pads at most 3 % more rows (the 32-row MFMA tiles it brings are worth that).  Column tile, among
// the variants of that height: the one with the smallest estimated makespan on 256 compute
// units -- rounds of workgroups times tile width -- with a 6 % handicap per halving of the
// width (narrow tiles re-read the packed weights more often per FLOP).  A mid-sized grid of a large
// problem may split its reduction (configure_ksplit): the estimate then takes the best split of each
// width, so that a wide tile in three slices can beat a narrow one that leaves the last round a third
// full (256 -> 384 channels, 3x3 at 13x13, backward data: 128x128 in 3 slices 325-334 us, 128x64
// unsplit 341).  Tiles that the patch-staged kernel may take (may_patch: the gather is one it can
// stage) are left out: that kernel does not split.
int32_t pick_corr_tile(int32_t rows, int64_t groups, int64_t ncols, int64_t kred, int64_t taps, bool may_patch) {
  int64_t best_pad = 0, best_bm = 0;
  for (int32_t t = 0; t < CORR_TILE_COUNT; ++t) {
    int32_t bm, bn, bk;
    corr_tile_shape(t, &bm, &bn, &bk);
    const int64_t pad = round_up(rows, bm);
    if (best_bm == 0 || pad < best_pad || (pad == best_pad && bm > best_bm)) {
      best_pad = pad;
      best_bm = bm;
    }
  }
  const int64_t min_pad = best_pad;
  for (int32_t t = 0; t < CORR_TILE_COUNT; ++t) {
    int32_t bm, bn, bk;
    corr_tile_shape(t, &bm, &bn, &bk);
    const int64_t pad = round_up(rows, bm);
    if (bm > best_bm && pad * 100 <= min_pad * 103) {
      best_pad = pad;
      best_bm = bm;
    }
  }
  int32_t best = -1;
  double best_cost = 0;
  for (int32_t t = 0; t < CORR_TILE_COUNT; ++t) {
    int32_t bm, bn, bk;
    corr_tile_shape(t, &bm, &bn, &bk);
    if (bm != best_bm) continue;
    const int64_t units = groups * (best_pad / bm) * ceil_div(ncols > 0 ? ncols : 1, bn);
    double cost = (double)ceil_div(units, 256) * bn;
    const int64_t chunks = ceil_div(kred, bk);
    const bool patch_tile = may_patch && ((bn == 256 && bm <= 48) || (taps >= 25 && bn == 128 && (bm == 128 || bm == 32)));
    if (units > 160 && units < 512 && !patch_tile && 2.0 * rows * (double)kred * (double)ncols * (double)groups >= 5e9)
      for (int64_t c = 2; c <= 8 && chunks / c >= 16; ++c) {  // the splits configure_ksplit may take
        const double split_cost = (double)ceil_div(units * c, 256) * bn / (double)c * (1.0 + 0.01 * (double)c);
        if (split_cost < cost) cost = split_cost;
      }
    for (int32_t w = bn; w < 256; w *= 2) cost *= 1.06;
    if (best < 0 || cost < best_cost) {
      best = t;
      best_cost = cost;
    }
  }
  return best;
}

// Thin groups.  The GEMM path pads a group's rows to 16 and its reduction to 16, so its cost per
// group is that of 16 x round_up(Cg*taps, 16) however few of them are real; the direct kernels cost
// Kg*Cg*taps multiply-adds per position at roughly a fifth of the matrix unit's rate for the 3x3 and
// 5x5 forms and a tenth for the general one (measured: 3x3 with 4 channels in and out per group is
// 1.8x faster direct, with 8 in and out 2x slower).
bool direct_is_faster(int64_t cg, int64_t kg, int64_t kh, int64_t kw) {
  const int64_t taps = kh * kw;
  const int64_t gemm = round_up(kg, 16) * round_up(cg * taps, 16);
  const bool rows_form = (kh == 3 && kw == 3) || (kh == 5 && kw == 5);
  return kg * cg * taps * (rows_form ? 5 : 10) <= gemm;
}

int32_t pick_wgrad_tile(int32_t rows, int32_t kred) {
  int32_t best = -1;
  int64_t best_work = 0, best_area = 0;
  for (int32_t t = 0; t < WGRAD_TILE_COUNT; ++t) {
    int32_t bm, bn, bk;
    wgrad_tile_shape(t, &bm, &bn, &bk);
    int64_t work = round_up(rows, bm) * round_up(kred, bn);
    const int64_t area = (int64_t)bm * bn;
    // a narrower tile must save at least 8 % of the padded work to be worth its extra LDS traffic
    if (best < 0 || work * 100 < best_work * 92 || (work <= best_work && area > best_area)) {
      best = t;
      best_work = work;
      best_area = area;
    }
  }
  return best;
}

// How the gather zeroes out-of-image elements (see corr_kernel): 0 = no padding at all and the blob
// below 2^31 bytes; 2 = at most 32 taps and the blob at most 2^29 bytes; 1 = anything else.
// `reach` = how far (bytes) a tap of a real column can point outside the blob: mode 2 adds
// 2^30 / 2^31 to such offsets and must neither wrap nor come back inside.
int32_t bounds_mode(bool no_padding, int64_t taps, int64_t bytes, int64_t reach) {
  if (no_padding && bytes < ((int64_t)1 << 31) - 4) return 0;
  if (taps <= 32 && bytes <= ((int64_t)1 << 29) && reach < ((int64_t)1 << 28)) return 2;
  return 1;
}

// One spatial dimension of the backward-data rewriting.  Input position x + pad = stride*a + r
// collects the taps i with i*dilation = stride*q + r from dy position a - q.
//  - Only the phases r in { i*dilation mod stride : i < kernel } are reached by any tap; when that
//    is a proper subset of 0 .. stride-1 of at most kMaxPhases values, the row space keeps only
//    those (a 1x1 stride-2 layer: one phase of four) and the rest of dx is zero-filled.
//  - When the stride divides the dilation (stride 1 included) the only phase is 0 and the taps sit
//    e = dilation/stride positions apart: kernel slots instead of (kernel-1)*dilation/stride + 1.
struct PhaseDim {
  int64_t Q, e, nv;
  int32_t tab;
  int32_t phase[kMaxPhases];
};

PhaseDim phase_dim(int64_t kernel, int64_t stride, int64_t dilation) {
  PhaseDim r = {};
  if (dilation % stride == 0) {
    r.Q = kernel;
    r.e = dilation / stride;
  } else {
    r.Q = (kernel - 1) * dilation / stride + 1;
    r.e = 1;
  }
  int64_t found = 0;
  int32_t vals[kMaxPhases];
  for (int64_t i = 0; i < kernel && found <= kMaxPhases; ++i) {
    const int32_t v = (int32_t)((i * dilation) % stride);
    bool seen = false;
    for (int64_t j = 0; j < found && j < kMaxPhases; ++j) seen = seen || vals[j] == v;
    if (!seen) {
      if (found < kMaxPhases) vals[found] = v;
      ++found;
    }
  }
  if (found >= stride || found > kMaxPhases) {  // every phase reached, or too many to tabulate
    r.nv = stride;
    r.tab = 0;
    return r;
  }
  for (int64_t i = 1; i < found; ++i)  // ascending order
    for (int64_t j = i; j > 0 && vals[j - 1] > vals[j]; --j) {
      const int32_t t = vals[j];
      vals[j] = vals[j - 1];
      vals[j - 1] = t;
    }
  r.nv = found;
  r.tab = 1;
  for (int64_t i = 0; i < found; ++i) r.phase[i] = vals[i];
  return r;
}

// "tile[m<bounds mode>,e<epilogue form>](S=<splits>,L=<launches>)", or "tile_patch[e.](S=1,L=2)" for the
// patch-staged kernel.
// Epilogue forms: s = separable byte offsets, r = range-checked stores with a compare per element,
// p = plain pointers (output of 2^31 bytes or more).
// L = kernel launches of the pass: the pack kernel, a zero fill (backward data with unreached
// phases), the main kernel, the reduce kernel of a split launch.
void corr_variant_name(char* buf, size_t len, int32_t tile, const CorrArgs& a, int zero_fill, int thin) {
  const char e = a.simple_epilogue ? 's' : ((uint32_t)a.out_elems < (1u << 29) ? 'r' : 'p');
  const int launches = 2 + (a.ksplit > 1) + (zero_fill != 0);
  if (thin && a.use_patch)  // rows staged in LDS, TW x TW taps unrolled, weights read in place: no pack kernel
    snprintf(buf, len, "corr_thin_r%d_lds%d[e%c](S=1,L=%d)", a.Mrows, a.TW, e, launches - 1);
  else if (thin)
    snprintf(buf, len, "corr_thin_r%d[m%d,e%c](S=1,L=%d)", a.Mrows, a.bounds_mode, e, launches);
  else if (a.use_patch)
    snprintf(buf, len, "%s_patch[e%c](S=%d,L=%d)", corr_tile_name(tile), e, a.ksplit, launches);
  else
    snprintf(buf, len, "%s[m%d,e%c](S=%d,L=%d)", corr_tile_name(tile), a.bounds_mode, e, a.ksplit, launches);
}

uint32_t koff_invalid(int32_t mode) { return mode == 0 ? 0x7FFFFFFCu : mode == 2 ? 0x40000000u : 0u; }

// Decides whether the patch-staged kernel runs this correlation and, if so, fills its fields.
// Used where the gather kernel's per-element work is largest: the 256-column tiles of at most 48 rows
// (measured: 5x5 grouped backward-data +9 %), and two 128-column tiles for kernels of 25 taps or more.
// Needs a stride-1, dilation-1 gather, 8-aligned channels per group, at least 3 taps, a blob of at
// most 2^30 bytes, and a patch that fits kPatchEPT*256 floats per channel and the LDS.
void configure_patch(CorrArgs& a, PackArgs& k, int64_t cg_in, int64_t n_img, int32_t bm, int32_t bn) {
  a.use_patch = 0;
  k.kperm_T = 0;
  const int64_t T = a.THW, TH = a.THW / a.TW;
  if (a.sh != 1 || a.sw != 1 || a.dh != 1 || a.dw != 1 || cg_in % 8 != 0 || T < 3) return;
  // 256-column tiles of at most 48 rows; with 25 taps or more also the 128x128 and 32x128 tiles, on grids
  // that the gather kernel would not split (measured with 5x5 kernels: 128x128 forward 451 -> 443 us,
  // 32x128 38 -> 34 us; with 3x3 kernels the gather kernel stays ahead, 298 -> 305 us)
  const bool wide = bn == 256 && bm <= 48;
  const bool many_taps = T >= 25 && bn == 128 && (bm == 128 || bm == 32) &&
                         (int64_t)a.G * a.m_tiles * a.col_tiles > 160;
  if (!wide && !many_taps) return;
  if ((int64_t)a.in_bytes > ((int64_t)1 << 30) || a.ncols < 1) return;
  const int64_t PH = a.P / a.PW, PWID = a.PW + a.TW - 1, RS = PH + TH - 1;
  // largest patch over all column tiles
  int64_t max_rows = 0;
  for (int64_t c0 = 0; c0 < a.ncols; c0 += bn) {
    const int64_t c1 = (c0 + bn < a.ncols ? c0 + bn : a.ncols) - 1;
    const int64_t n0 = c0 / a.P, a0 = (c0 % a.P) / a.PW, n1 = c1 / a.P, a1 = (c1 % a.P) / a.PW;
    const int64_t R0 = PH - a0 + TH - 1;
    const int64_t rows = (n1 == n0 ? a1 - a0 : R0 + (n1 - n0 - 1) * RS + a1) + TH;
    if (rows > max_rows) max_rows = rows;
  }
  // Channel stride of the patch in LDS.  At one MFMA step the four lane groups of a wave read four
  // channels 2*psz floats apart, 16 consecutive positions each: a stride of 8 mod 16 puts those
  // four runs on different banks.
  int64_t psz = max_rows * PWID;
  psz += (8 - psz % 16 + 16) % 16;
  const int64_t lds = (2 * (int64_t)bm * 20 + 16 * psz) * 4;
  if (psz > kPatchEPT * 256 || lds > 80 * 1024 || lds < 16 * ((int64_t)bm + bn)) return;
  a.use_patch = 1;
  a.Cg_in = (int32_t)cg_in;
  a.NS = (int32_t)(cg_in / 8 * T);
  a.PH = (int32_t)PH;
  a.Nimg = (int32_t)n_img;
  a.PWID = (int32_t)PWID;
  a.PSZ = (int32_t)psz;
  a.mPWID = make_magic((uint32_t)PWID);
  a.mRSEG = make_magic((uint32_t)RS);
  k.kperm_T = (int32_t)T;
}

// Split of the reduction: with few workgroups and a long chunk loop the chip idles while each
// workgroup walks its chunks one barrier at a time; S slices run side by side and a reduce kernel
// adds them.  Worth an extra launch when the grid is well under one workgroup per compute unit,
// or when a large problem leaves the compute units unevenly loaded.
// bm x bn: the tile; elem_bytes: 4 or 8 (the double path runs the same rule on its own tiles).
void configure_ksplit(CorrArgs& a, int64_t out_elems, int32_t bm, int32_t bn, int32_t elem_bytes = 4) {
  a.ksplit = 1;
  a.chunks_per_split = a.KP / 16;
  a.out_elems = (int32_t)out_elems;
  a.simple_epilogue = a.RShw == 1 && a.tab_h == 0 && a.tab_w == 0 && 4 * out_elems <= ((int64_t)1 << 30);
  const int64_t units = (int64_t)a.G * a.m_tiles * a.col_tiles, chunks = a.KP / 16;
  if (a.use_patch || chunks < 8 || a.ncols < 1) return;
  int64_t S = 1;
  const double flops = 2.0 * a.Mrows * a.Kred * (double)a.ncols * a.G;
  if (units <= 160 && flops < 2e9) {
    // Small grid of a small problem: the number of slices with the smallest modelled time.  A
    // workgroup that has its compute unit to itself walks its chunks at the latency of one chunk --
    // 0.18 us plus 0.30 us per 4096 tile elements (twice that in doubles) -- and S slices cost the
    // reduce kernel's launch, 1.6 us, plus their partial sums written and read once at 2.4 TB/s
    // (0.83 us per MB).  Constants fitted to split sweeps of the nine such passes of the benchmark's
    // small layers (rms error 1 us; the model picks the fastest or second fastest S on each: 2.a
    // forward, 32 chunks on 64 tiles of 64x64, 0.8 MB out: 4 slices 13.4 us against 14.6 with 8 and
    // 21.7 unsplit; 3.a forward, 16 chunks on 100 tiles, 1.6 MB out: unsplit 14.4 us against 18.0
    // with 4).  At most 16 slices of at least two chunks, at most 1024 workgroups.
    const double t_chunk = 0.18 + 0.30 * (elem_bytes == 8 ? 2.0 : 1.0) * (double)(bm * bn) / 4096.0;
    const double out_mb = (double)out_elems * elem_bytes / 1e6;
    double best_t = (double)chunks * t_chunk;
    for (int64_t c = 2; c <= 16 && c <= chunks / 2 && units * c <= 1024; ++c) {
      const double t = (double)ceil_div(chunks, c) * t_chunk + 1.6 + 0.83 * (double)c * out_mb;
      if (t < best_t) {
        best_t = t;
        S = c;
      }
    }
  } else if (units <= 160) {
    // Small grid of a larger problem (the matrix pipes, not latency, set the pace once the slices
    // fill the chip): two workgroups per compute unit, at least four chunks per slice
    S = ceil_div(512, units);
    if (S > chunks / 4) S = chunks / 4;
    if (S > 16) S = 16;
    // a long reduction carries twice as many slices as long as each keeps 32 chunks (the 9216 -> 4096
    // InnerProduct backward-data pass: 144 tiles, 256 chunks, 4 -> 8 slices, 118 -> 105 us)
    int64_t S2 = ceil_div(1024, units);
    if (S2 > chunks / 32) S2 = chunks / 32;
    if (S2 > 16) S2 = 16;
    if (S2 > S) S = S2;
  } else if (units < 512 && flops >= 5e9) {
    // Mid-sized grids of a large problem (a 14x14 or 7x7 layer with hundreds of channels): one or
    // two workgroups per compute unit with some units idle.  Take the split that brings the load
    // of the busiest unit, relative to the unsplit grid, down by at least 15 % (20 % when the
    // unsplit grid already has two workgroups on some units; 1 % per slice charged for the partial
    // sums); every slice keeps at least 16 chunks.
    const double base = (double)ceil_div(units, 256);
    double best = base > 1.0 ? 0.80 : 0.85;
    for (int64_t c = 2; c <= 8 && chunks / c >= 16; ++c) {
      const double ratio = (double)ceil_div(units * c, 256) / ((double)c * base) * (1.0 + 0.01 * (double)c);
      if (ratio < best) {
        best = ratio;
        S = c;
      }
    }
  }
  if (S < 2) return;
  a.chunks_per_split = (int32_t)ceil_div(chunks, S);
  a.ksplit = (int32_t)ceil_div(chunks, a.chunks_per_split);
}

// GEMMs of at most four rows per group (backward data of a layer with one to four input channels
// per group at stride 1, forward with that few outputs) with the offset-only epilogue take
// corr_thin_kernel: one lane per column, scalar A operands, no matrix unit -- the 16-row tiles
// spend three quarters or more of their matrix instructions on padding there.  The packed operand
// and the k table stay as they are (natural k order); the reduction is not split.
int32_t configure_thin(CorrArgs& a, PackArgs& k, int64_t cg_in, int64_t n_img, bool backward) {
  if (a.Mrows > 4 || !a.simple_epilogue || a.ncols < 1) return 0;
  a.use_patch = 0;
  k.kperm_T = 0;
  a.ksplit = 1;
  a.chunks_per_split = a.KP / 16;
  // A stride-1, dilation-1 gather with 3x3 or 5x5 taps whose rows fit LDS takes the staged form: 128
  // columns per workgroup, all channels of the group at once, the patch of the largest tile (geometry
  // of configure_patch) at most 512 floats per channel and 64 KB in all.  It reads its A operands
  // from the weight blob (output channel, input channel, tap): forward rows are output channels and
  // the gathered channels inputs; backward data the other way round with the taps reversed.
  const int64_t T = a.THW, w_grp = (int64_t)a.Mrows * cg_in * T;
  if (a.sh == 1 && a.sw == 1 && a.dh == 1 && a.dw == 1 && (a.TW == 3 || a.TW == 5) && T == a.TW * a.TW &&
      (int64_t)a.in_bytes <= ((int64_t)1 << 30) && w_grp * a.G < ((int64_t)1 << 31)) {
    const int64_t bn = 128, TH = a.TW;
    const int64_t PH = a.P / a.PW, PWID = a.PW + a.TW - 1, RS = PH + TH - 1;
    int64_t max_rows = 0;
    for (int64_t c0 = 0; c0 < a.ncols; c0 += bn) {
      const int64_t c1 = (c0 + bn < a.ncols ? c0 + bn : a.ncols) - 1;
      const int64_t n0 = c0 / a.P, a0 = (c0 % a.P) / a.PW, n1 = c1 / a.P, a1 = (c1 % a.P) / a.PW;
      const int64_t R0 = PH - a0 + TH - 1;
      const int64_t rows = (n1 == n0 ? a1 - a0 : R0 + (n1 - n0 - 1) * RS + a1) + TH;
      if (rows > max_rows) max_rows = rows;
    }
    const int64_t psz = max_rows * PWID;
    if (psz <= 512 && cg_in * psz * 4 <= 64 * 1024) {
      a.use_patch = 1;
      a.Cg_in = (int32_t)cg_in;
      a.NS = 0;
      a.PH = (int32_t)PH;
      a.Nimg = (int32_t)n_img;
      a.PWID = (int32_t)PWID;
      a.PSZ = (int32_t)psz;
      a.mPWID = make_magic((uint32_t)PWID);
      a.mRSEG = make_magic((uint32_t)RS);
      a.w_grp_stride = (int32_t)w_grp;
      a.w_row_stride = (int32_t)(backward ? T : cg_in * T);
      a.w_chan_stride = (int32_t)(backward ? a.Mrows * T : T);
      a.w_reversed = backward ? 1 : 0;
    }
  }
  return 1;
}

}  // namespace

namespace mi355conv {

int record_hip_error(int e) {
  g_last_hip_error = e;
  return CONV_EHIP;
}

int conv_desc_backward_filter_workspace_bytes(const conv_desc* d, size_t* bytes) {
  if (!d || !bytes) return CONV_EINVAL;
  *bytes = d->wg_ws;
  return CONV_OK;
}

int run_forward(const conv_desc* d, const float* x, const float* w, const float* bias, float* y, void* ws,
                size_t ws_bytes, void* hip_stream) {
  if (!d || !w) return CONV_EINVAL;
  if ((d->p.bias_term != 0) != (bias != nullptr)) return CONV_EINVAL;
  if (d->p.n == 0) return CONV_OK;  // empty blobs: nothing to read or write
  if (!x || !y) return CONV_EINVAL;
  if (d->use_direct) {
    DirectArgs da = d->dir;
    da.in = x;
    da.w = w;
    da.bias = bias;
    da.out = y;
    const int ed = launch_direct(0, da, false, hip_stream);
    return ed ? record_hip_error(ed) : CONV_OK;
  }
  if (d->fwd_ws > 0 && (!ws || ws_bytes < d->fwd_ws)) return CONV_EWORKSPACE;
  PackArgs k = d->fwd_pack;
  k.w = w;
  k.A = static_cast<float*>(ws);
  k.ktab = reinterpret_cast<KTabEntry*>(k.A + (size_t)k.G * k.KP * k.MP);
  const bool in_place = d->fwd_thin && d->fwd.use_patch;  // that kernel reads the weight blob itself
  int e = in_place ? 0 : launch_pack(k, hip_stream);
  if (e) return record_hip_error(e);
  CorrArgs a = d->fwd;
  a.A = in_place ? w : k.A;
  a.ktab = k.ktab;
  a.in = x;
  a.bias = bias;
  a.out = y;
  a.part = reinterpret_cast<float*>(static_cast<char*>(ws) + d->fwd_pack_bytes);
  e = d->fwd_thin    ? launch_corr_thin(a, hip_stream)
      : a.use_patch ? launch_corr_patch(d->fwd_tile, a, hip_stream)
                    : launch_corr(d->fwd_tile, a, hip_stream);
  if (e) return record_hip_error(e);
  if (a.ksplit > 1) {  // add the split partials and the bias
    ReduceArgs r = {};
    r.part = a.part;
    r.dst = y;
    r.count = a.out_elems;
    r.S = a.ksplit;
    r.beta = 0.f;
    r.bias = bias;
    r.chan_elems = d->OH * d->OW;
    r.channels = d->p.num_output;
    r.mChanElems = make_magic(r.chan_elems);
    r.mChannels = make_magic(r.channels);
    e = launch_reduce(r, hip_stream);
  }
  return e ? record_hip_error(e) : CONV_OK;
}

int run_backward_data(const conv_desc* d, const float* w, const float* dy, float* dx, float beta, void* ws,
                      size_t ws_bytes, void* hip_stream) {
  if (!d || !w) return CONV_EINVAL;
  if (!(beta == 0.f || beta == 1.f)) return CONV_EINVAL;
  if (d->p.n == 0) return CONV_OK;
  if (!dy || !dx) return CONV_EINVAL;
  if (d->use_direct) {
    DirectArgs da = d->dir;
    da.in = dy;
    da.w = w;
    da.out = dx;
    if (beta != 0.f) return CONV_EINVAL;  // accumulation into dx is only used by the ungrouped InnerProduct passes
    const int ed = launch_direct(1, da, false, hip_stream);
    return ed ? record_hip_error(ed) : CONV_OK;
  }
  if (d->bwd_ws > 0 && (!ws || ws_bytes < d->bwd_ws)) return CONV_EWORKSPACE;
  PackArgs k = d->bwd_pack;
  k.w = w;
  k.A = static_cast<float*>(ws);
  k.ktab = reinterpret_cast<KTabEntry*>(k.A + (size_t)k.G * k.KP * k.MP);
  const bool in_place = d->bwd_thin && d->bwd.use_patch;  // that kernel reads the weight blob itself
  int e = in_place ? 0 : launch_pack(k, hip_stream);
  if (e) return record_hip_error(e);
  CorrArgs a = d->bwd;
  a.A = in_place ? w : k.A;
  a.ktab = k.ktab;
  a.in = dy;
  a.bias = nullptr;
  a.out = dx;
  a.accumulate = beta != 0.f;
  a.part = reinterpret_cast<float*>(static_cast<char*>(ws) + d->bwd_pack_bytes);
  if (d->bwd_zero_fill) {  // positions no tap reaches: zero the split partials, or dx itself when it is overwritten
    if (a.ksplit > 1)
      e = launch_fill_zero(a.part, (size_t)a.ksplit * a.out_elems * 4, hip_stream);
    else if (beta == 0.f)
      e = launch_fill_zero(dx, (size_t)a.out_elems * 4, hip_stream);
    if (e) return record_hip_error(e);
  }
  e = d->bwd_thin    ? launch_corr_thin(a, hip_stream)
      : a.use_patch ? launch_corr_patch(d->bwd_tile, a, hip_stream)
                    : launch_corr(d->bwd_tile, a, hip_stream);
  if (e) return record_hip_error(e);
  if (a.ksplit > 1) {
    ReduceArgs r = {};
    r.part = a.part;
    r.dst = dx;
    r.count = a.out_elems;
    r.S = a.ksplit;
    r.beta = beta;
    e = launch_reduce(r, hip_stream);
  }
  return e ? record_hip_error(e) : CONV_OK;
}

int run_backward_filter(const conv_desc* d, const float* x, const float* dy, float* dw, float beta, void* ws,
                        size_t ws_bytes, void* hip_stream, const ReduceExtras& extras, float* db) {
  if (!d || !dw) return CONV_EINVAL;
  if (!(beta == 0.f || beta == 1.f)) return CONV_EINVAL;
  const bool empty = d->p.n == 0;  // the gradient sum is empty: dw = beta*dw
  if (!empty && (!x || !dy)) return CONV_EINVAL;
  const size_t need = db ? d->wgb_ws : d->wg_ws;
  if (!empty && need > 0 && (!ws || ws_bytes < need)) return CONV_EWORKSPACE;
  const int32_t w_elems = (int32_t)((int64_t)d->p.num_output * d->wg.Kred);
  WgradArgs a = d->wg;
  a.dy = dy;
  a.x = x;
  a.part = static_cast<float*>(ws);
  int e = 0;
  if (d->use_direct) {
    // thin groups: the direct filter-gradient kernel; its workgroups of a group's first input channel
    // also add up the dy values they read (S x K sums behind the filter partials)
    DirectArgs da = d->dir;
    da.in = x;
    da.w = dy;
    da.part = ws;
    a.S = da.S;
    a.n_tiles = 1;
    if (db) da.bias_part = a.bias_part = a.part + (size_t)da.S * w_elems;
    if (!empty) e = launch_direct(2, da, false, hip_stream);
  } else if (!empty) {
    if (db) a.bias_part = a.part + (size_t)a.S * w_elems;  // row sums of dy ride along, behind the filter partials
    e = launch_wgrad(d->wg_tile, a, hip_stream);
  }
  if (e) return record_hip_error(e);
  ReduceArgs r = {};
  r.part = a.part;
  r.dst = dw;
  r.count = w_elems;
  r.S = empty ? 0 : a.S;
  r.beta = beta;
  r.bias = extras.bias;
  r.chan_elems = extras.chan_elems;
  r.channels = extras.channels;
  r.mChanElems = make_magic(r.chan_elems);
  r.mChannels = make_magic(r.channels);
  r.relu = extras.relu;
  if (db) {  // the same launch finishes db from the S * n_tiles shares of the row sums
    r.part2 = empty ? nullptr : a.bias_part;
    r.dst2 = db;
    r.count2 = d->p.num_output;
    r.S2 = empty ? 0 : a.S * a.n_tiles;
  }
  e = launch_reduce(r, hip_stream);
  return e ? record_hip_error(e) : CONV_OK;
}

}  // namespace mi355conv

extern "C" {

int conv_desc_create(conv_desc_t** out, const conv_params_t* pp) {
  if (!out || !pp) return CONV_EINVAL;
  const conv_params_t p = *pp;
  if (p.n < 0 || p.c < 1 || p.h < 1 || p.w < 1 || p.num_output < 1) return CONV_EINVAL;
  if (p.kernel_h < 1 || p.kernel_w < 1 || p.stride_h < 1 || p.stride_w < 1) return CONV_EINVAL;
  if (p.pad_h < 0 || p.pad_w < 0 || p.dilation_h < 1 || p.dilation_w < 1) return CONV_EINVAL;
  if (p.group < 1 || p.c % p.group != 0 || p.num_output % p.group != 0) return CONV_EINVAL;
  if (p.bias_term != 0 && p.bias_term != 1) return CONV_EINVAL;

  const int64_t ext_h = (int64_t)p.dilation_h * (p.kernel_h - 1) + 1;
  const int64_t ext_w = (int64_t)p.dilation_w * (p.kernel_w - 1) + 1;
  const int64_t OH = floor_div((int64_t)p.h + 2 * (int64_t)p.pad_h - ext_h, p.stride_h) + 1;
  const int64_t OW = floor_div((int64_t)p.w + 2 * (int64_t)p.pad_w - ext_w, p.stride_w) + 1;
  if (OH < 1 || OW < 1) return CONV_ESHAPE;
  // tap offsets are packed into 16 bits, coordinates into 28
  if (ext_h > 32768 || ext_w > 32768 || p.pad_h > (1 << 20) || p.pad_w > (1 << 20)) return CONV_ESHAPE;
  if (p.h > (1 << 24) || p.w > (1 << 24) || p.stride_h > (1 << 20) || p.stride_w > (1 << 20)) return CONV_ESHAPE;

  const int64_t N = p.n, C = p.c, H = p.h, W = p.w, K = p.num_output, G = p.group;
  const int64_t Cg = C / G, Kg = K / G;
  const int64_t kred = Cg * p.kernel_h * p.kernel_w;
  // sizes in 128-bit arithmetic first: four 31-bit factors do not fit 64 bits
  const __int128 big = kMaxElems;
  if ((__int128)C * H * W >= big || (__int128)K * OH * OW >= big || (__int128)N * C * H * W >= big ||
      (__int128)N * K * OH * OW >= big || (__int128)K * Cg * p.kernel_h * p.kernel_w >= big)
    return CONV_ESHAPE;
  const int64_t x_elems = N * C * H * W, y_elems = N * K * OH * OW, w_elems = K * kred;

  conv_desc* d = new (std::nothrow) conv_desc;
  if (!d) return CONV_EINVAL;
  memset(d, 0, sizeof(*d));
  d->p = p;
  d->OH = (int32_t)OH;
  d->OW = (int32_t)OW;
  d->Cg = (int32_t)Cg;
  d->Kg = (int32_t)Kg;

  int32_t bm, bn, bk;

  // ---- forward: rows = output channels of a group, k = (c, i, j), columns = (n, oh, ow) ----
  {
    d->fwd_tile = pick_corr_tile((int32_t)Kg, G, N * OH * OW, kred, (int64_t)p.kernel_h * p.kernel_w,
                                 p.stride_h == 1 && p.stride_w == 1 && p.dilation_h == 1 && p.dilation_w == 1 && Cg % 8 == 0);
    corr_tile_shape(d->fwd_tile, &bm, &bn, &bk);
    CorrArgs& a = d->fwd;
    a.ncols = (int32_t)(N * OH * OW);
    a.P = (int32_t)(OH * OW);
    a.PW = (int32_t)OW;
    a.mP = make_magic(a.P);
    a.mPW = make_magic(a.PW);
    a.IH = p.h;
    a.IW = p.w;
    a.IHW = p.h * p.w;
    a.in_img_stride = (int32_t)(C * H * W);
    a.in_grp_stride = (int32_t)(Cg * H * W);
    a.in_bytes = (uint32_t)(4 * x_elems);
    a.bounds_mode = bounds_mode(p.pad_h == 0 && p.pad_w == 0, (int64_t)p.kernel_h * p.kernel_w, 4 * x_elems,
                                4 * ((p.pad_h + ext_h) * W + p.pad_w + ext_w));
    a.TW = p.kernel_w;
    a.THW = p.kernel_h * p.kernel_w;
    a.mTW = make_magic(a.TW);
    a.mTHW = make_magic(a.THW);
    a.sh = p.stride_h;
    a.sw = p.stride_w;
    a.dh = p.dilation_h;
    a.dw = p.dilation_w;
    a.ph = p.pad_h;
    a.pw = p.pad_w;
    a.Kred = (int32_t)kred;
    a.KP = (int32_t)round_up(kred, bk);
    a.Mrows = (int32_t)Kg;
    a.MP = (int32_t)round_up(Kg, bm);
    a.RSh = a.RSw = a.RShw = 1;
    a.OSh = a.OSw = 1;
    a.mRSw = make_magic(1);
    a.mRShw = make_magic(1);
    a.opad_h = a.opad_w = 0;
    a.OHd = (int32_t)OH;
    a.OWd = (int32_t)OW;
    a.out_img_stride = (int32_t)(K * OH * OW);
    a.chan_per_grp = (int32_t)Kg;
    a.G = (int32_t)G;
    a.m_tiles = a.MP / bm;
    a.col_tiles = (int32_t)ceil_div(a.ncols, bn);
    PackArgs& k = d->fwd_pack;
    k.mode = 0;
    k.G = (int32_t)G;
    k.Kg = (int32_t)Kg;
    k.Cg = (int32_t)Cg;
    k.kh = p.kernel_h;
    k.kw = p.kernel_w;
    k.sh = k.sw = k.dh = k.dw = 1;
    k.Qh = k.Qw = 1;
    k.Kred = a.Kred;
    k.KP = a.KP;
    k.Mrows = a.Mrows;
    k.MP = a.MP;
    k.tTW = a.TW;
    k.tTHW = a.THW;
    k.tIW = a.IW;
    k.tIHW = a.IHW;
    k.tdh = a.dh;
    k.tdw = a.dw;
    k.koff_invalid = koff_invalid(a.bounds_mode);
    configure_patch(a, k, Cg, N, bm, bn);
    configure_ksplit(a, y_elems, bm, bn);
    d->fwd_thin = configure_thin(a, k, Cg, N, false);
    const int64_t pack_elems = G * (int64_t)a.KP * a.MP;
    if (pack_elems >= kMaxElems || (int64_t)G * a.m_tiles * a.col_tiles >= ((int64_t)1 << 31)) {
      delete d;
      return CONV_ESHAPE;
    }
    d->fwd_pack_bytes = (size_t)pack_elems * 4 + (size_t)a.KP * sizeof(KTabEntry);
    d->fwd_ws = d->fwd_pack_bytes + (a.ksplit > 1 ? (size_t)a.ksplit * y_elems * 4 : 0);
  }

  // ---- backward data: a stride-1 correlation over dy whose rows are (c, row phase, column
  // phase) of dx -- input position h + pad = stride*a + rh collects the taps i with
  // i*dilation = stride*q + rh from dy row a - q (see phase_dim for the tap slots and the phases
  // kept).  Positions with a < a0 = pad / stride lie wholly in the padding, so the column space
  // starts at a0. ----
  {
    const PhaseDim dim_h = phase_dim(p.kernel_h, p.stride_h, p.dilation_h);
    const PhaseDim dim_w = phase_dim(p.kernel_w, p.stride_w, p.dilation_w);
    const int64_t Qh = dim_h.Q, Qw = dim_w.Q;
    const int64_t a0h = p.pad_h / p.stride_h, a0w = p.pad_w / p.stride_w;
    const int64_t Ah = (H - 1 + p.pad_h) / p.stride_h + 1 - a0h;
    const int64_t Aw = (W - 1 + p.pad_w) / p.stride_w + 1 - a0w;
    const int64_t rows = Cg * dim_h.nv * dim_w.nv;
    const int64_t kred_b = Kg * Qh * Qw;
    d->bwd_zero_fill = dim_h.nv < p.stride_h || dim_w.nv < p.stride_w;
    if (rows >= ((int64_t)1 << 24) || N * Ah * Aw >= ((int64_t)1 << 31) || kred_b >= kMaxElems) {
      delete d;
      return CONV_ESHAPE;
    }
    d->bwd_tile = pick_corr_tile((int32_t)rows, G, N * Ah * Aw, kred_b, Qh * Qw, Kg % 8 == 0);
    corr_tile_shape(d->bwd_tile, &bm, &bn, &bk);
    CorrArgs& a = d->bwd;
    a.ncols = (int32_t)(N * Ah * Aw);
    a.P = (int32_t)(Ah * Aw);
    a.PW = (int32_t)Aw;
    a.mP = make_magic(a.P);
    a.mPW = make_magic(a.PW);
    a.IH = (int32_t)OH;
    a.IW = (int32_t)OW;
    a.IHW = (int32_t)(OH * OW);
    a.in_img_stride = (int32_t)(K * OH * OW);
    a.in_grp_stride = (int32_t)(Kg * OH * OW);
    a.in_bytes = (uint32_t)(4 * y_elems);
    a.bounds_mode = bounds_mode(false, Qh * Qw, 4 * y_elems,
                                4 * (2 * ((Qh - 1) * dim_h.e + 1) * OW + 2 * ((Qw - 1) * dim_w.e + 1)));
    a.TW = (int32_t)Qw;
    a.THW = (int32_t)(Qh * Qw);
    a.mTW = make_magic(a.TW);
    a.mTHW = make_magic(a.THW);
    a.sh = a.sw = 1;
    a.dh = (int32_t)dim_h.e;
    a.dw = (int32_t)dim_w.e;
    a.ph = (int32_t)((Qh - 1) * dim_h.e - a0h);
    a.pw = (int32_t)((Qw - 1) * dim_w.e - a0w);
    a.Kred = (int32_t)kred_b;
    a.KP = (int32_t)round_up(kred_b, bk);
    a.Mrows = (int32_t)rows;
    a.MP = (int32_t)round_up(rows, bm);
    a.RSh = (int32_t)dim_h.nv;
    a.RSw = (int32_t)dim_w.nv;
    a.RShw = a.RSh * a.RSw;
    a.mRSw = make_magic(a.RSw);
    a.mRShw = make_magic(a.RShw);
    a.OSh = p.stride_h;
    a.OSw = p.stride_w;
    a.tab_h = dim_h.tab;
    a.tab_w = dim_w.tab;
    for (int i = 0; i < kMaxPhases; ++i) {
      a.phase_h[i] = dim_h.phase[i];
      a.phase_w[i] = dim_w.phase[i];
    }
    a.opad_h = (int32_t)(p.pad_h - a0h * p.stride_h);
    a.opad_w = (int32_t)(p.pad_w - a0w * p.stride_w);
    a.OHd = p.h;
    a.OWd = p.w;
    a.out_img_stride = (int32_t)(C * H * W);
    a.chan_per_grp = (int32_t)Cg;
    a.G = (int32_t)G;
    a.m_tiles = a.MP / bm;
    a.col_tiles = (int32_t)ceil_div(a.ncols, bn);
    PackArgs& k = d->bwd_pack;
    k.mode = 1;
    k.G = (int32_t)G;
    k.Kg = (int32_t)Kg;
    k.Cg = (int32_t)Cg;
    k.kh = p.kernel_h;
    k.kw = p.kernel_w;
    k.sh = p.stride_h;
    k.sw = p.stride_w;
    k.dh = p.dilation_h;
    k.dw = p.dilation_w;
    k.Qh = (int32_t)Qh;
    k.Qw = (int32_t)Qw;
    k.nvh = a.RSh;
    k.nvw = a.RSw;
    k.eh = a.dh;
    k.ew = a.dw;
    k.tab_h = a.tab_h;
    k.tab_w = a.tab_w;
    for (int i = 0; i < kMaxPhases; ++i) {
      k.phase_h[i] = a.phase_h[i];
      k.phase_w[i] = a.phase_w[i];
    }
    k.Kred = a.Kred;
    k.KP = a.KP;
    k.Mrows = a.Mrows;
    k.MP = a.MP;
    k.tTW = a.TW;
    k.tTHW = a.THW;
    k.tIW = a.IW;
    k.tIHW = a.IHW;
    k.tdh = a.dh;
    k.tdw = a.dw;
    k.koff_invalid = koff_invalid(a.bounds_mode);
    configure_patch(a, k, Kg, N, bm, bn);
    configure_ksplit(a, x_elems, bm, bn);
    d->bwd_thin = configure_thin(a, k, Kg, N, true);
    const int64_t pack_elems = G * (int64_t)a.KP * a.MP;
    if (pack_elems >= kMaxElems || (int64_t)G * a.m_tiles * a.col_tiles >= ((int64_t)1 << 31)) {
      delete d;
      return CONV_ESHAPE;
    }
    d->bwd_pack_bytes = (size_t)pack_elems * 4 + (size_t)a.KP * sizeof(KTabEntry);
    d->bwd_ws = d->bwd_pack_bytes + (a.ksplit > 1 ? (size_t)a.ksplit * x_elems * 4 : 0);
  }

  // ---- backward filter: rows = output channels, columns = (c, i, j), reduction over (n, oh, ow)
  {
    d->wg_tile = pick_wgrad_tile((int32_t)Kg, (int32_t)kred);
    wgrad_tile_shape(d->wg_tile, &bm, &bn, &bk);
    WgradArgs& a = d->wg;
    a.ncols = (int32_t)(N * OH * OW);
    a.P = (int32_t)(OH * OW);
    a.PW = (int32_t)OW;
    a.mP = make_magic(a.P);
    a.mPW = make_magic(a.PW);
    a.dy_bytes = (uint32_t)(4 * y_elems);
    a.x_bytes = (uint32_t)(4 * x_elems);
    // the dy base of a column past the split is 2^31: both blobs must stay below that for modes 0 and 2
    a.bounds_mode = 1;
    if (4 * y_elems < ((int64_t)1 << 31) - 4) {
      a.bounds_mode = bounds_mode(p.pad_h == 0 && p.pad_w == 0, (int64_t)p.kernel_h * p.kernel_w, 4 * x_elems,
                                  4 * ((p.pad_h + ext_h) * W + p.pad_w + ext_w));
      if (a.bounds_mode == 2 && (p.dilation_h != 1 || p.dilation_w != 1 || p.kernel_h * p.kernel_w > 31))
        a.bounds_mode = 1;
    }
    a.Kg = (int32_t)Kg;
    a.Ktot = (int32_t)K;
    a.Cg = (int32_t)Cg;
    a.C = p.c;
    a.H = p.h;
    a.W = p.w;
    a.HW = p.h * p.w;
    a.kw = p.kernel_w;
    a.khw = p.kernel_h * p.kernel_w;
    a.mKW = make_magic(a.kw);
    a.mKHW = make_magic(a.khw);
    a.sh = p.stride_h;
    a.sw = p.stride_w;
    a.dh = p.dilation_h;
    a.dw = p.dilation_w;
    a.ph = p.pad_h;
    a.pw = p.pad_w;
    a.Kred = (int32_t)kred;
    a.G = (int32_t)G;
    a.m_tiles = (int32_t)ceil_div(Kg, bm);
    a.n_tiles = (int32_t)ceil_div(kred, bn);
    // Split the reduction so that the whole grid is resident at once -- LDS holds two workgroups per
    // compute unit (three of the 32-row tile), and a grid of 1.4 times that many runs a second,
    // mostly empty round (5.a: 714 workgroups on 512 places took 255 us, 507 take 234) -- with each
    // split at least four k tiles long and the partials at most 32 MiB; a grid slightly above a
    // multiple of the 256 compute units is trimmed back to it (its last few workgroups would
    // otherwise share a compute unit while the others have one to themselves).
    const int64_t max_by_len = ceil_div((int64_t)a.ncols, 4 * bk);
    const int64_t max_by_ws = ((int64_t)8 << 20) / (w_elems > 0 ? w_elems : 1);
    auto splits_for = [&](int64_t tiles, int64_t places) {
      int64_t S = places / tiles;
      if (S > max_by_len) S = max_by_len;
      if (S > max_by_ws) S = max_by_ws;
      if (S > 256) S = 256;  // beyond one split per compute unit the reduce kernel only gets slower
      if (S < 1) S = 1;
      while (S > 1 && tiles * S > 256 && (tiles * S) % 256 != 0 && (tiles * S) % 256 < 64) --S;
      return S;
    };
    int64_t tiles = G * a.m_tiles * a.n_tiles;
    int64_t S = splits_for(tiles, 256 * (bm == 32 ? 3 : 2));
    // A grid that cannot fill the compute units because its splits are as short as they may get takes
    // the 32-row tile instead of the 64-row one when both pad the rows alike: twice the workgroups,
    // three resident per compute unit (2.a 12.9 -> 10.8 us, 3.b 13.2 -> 11.0, 3.c 12.3 -> 10.1).
    if (d->wg_tile == WGRAD_64x128 && tiles * S < 256 && round_up(Kg, 32) == round_up(Kg, 64)) {
      d->wg_tile = WGRAD_32x128;
      wgrad_tile_shape(d->wg_tile, &bm, &bn, &bk);
      a.m_tiles = (int32_t)ceil_div(Kg, bm);
      a.n_tiles = (int32_t)ceil_div(kred, bn);
      tiles = G * a.m_tiles * a.n_tiles;
      S = splits_for(tiles, 256 * 3);
    }
    a.cols_per_split = (int32_t)round_up(ceil_div((int64_t)a.ncols > 0 ? a.ncols : 1, S), bk);
    a.S = (int32_t)ceil_div((int64_t)a.ncols > 0 ? a.ncols : 1, a.cols_per_split);
    if (a.S * w_elems >= kMaxElems || tiles * a.S >= ((int64_t)1 << 31)) {
      delete d;
      return CONV_ESHAPE;
    }
    a.part_stride = (int32_t)w_elems;
    a.bias_part = nullptr;
    d->wg_ws = (size_t)a.S * (size_t)w_elems * 4;
    d->wgb_ws = (size_t)a.S * (size_t)(w_elems + a.n_tiles * K) * 4;
    if (a.S * (w_elems + a.n_tiles * K) >= kMaxElems) {
      delete d;
      return CONV_ESHAPE;
    }
  }

  // ---- backward bias ----
  {
    BiasGradArgs& a = d->bg;
    a.N = p.n;
    a.K = p.num_output;
    a.P = (int32_t)(OH * OW);
    int64_t S = ceil_div(2048, K);
    if (S > N) S = N;
    if (S < 1) S = 1;
    // up to a megabyte: one workgroup per channel sums the whole batch and finishes db
    // itself -- the second launch would cost more than the lost parallelism
    d->bg_direct = y_elems * 4 <= ((int64_t)1 << 20);
    if (d->bg_direct) S = 1;
    a.n_per_split = (int32_t)ceil_div(N > 0 ? N : 1, S);
    a.S = (int32_t)ceil_div(N > 0 ? N : 1, a.n_per_split);
    d->bg_ws = p.bias_term ? (size_t)a.S * K * 4 : 0;
  }

  // ---- double base type: the same geometry on the fp64 tiles, compare-style bounds checks ----
  {
    const int32_t bn64 = kF64TileCols, bk64 = kF64TileK;
    const int64_t max64 = (int64_t)1 << 29;  // 32-bit byte offsets of 8-byte elements
    d->f64_ok = x_elems < max64 && y_elems < max64 && w_elems < max64;
    auto corr64 = [&](const CorrArgs& src, const PackArgs& psrc, CorrArgs& a, PackArgs& k, int64_t in_elems,
                      size_t& ws, int32_t& tile_rows) {
      a = src;
      const int32_t bm64 = tile_rows = f64_pick_rows(src.Mrows, false);
      a.in_bytes = (uint32_t)(8 * in_elems);
      a.bounds_mode = 1;
      a.KP = (int32_t)round_up(a.Kred, bk64);
      a.MP = (int32_t)round_up(a.Mrows, bm64);
      a.m_tiles = a.MP / bm64;
      a.col_tiles = (int32_t)ceil_div(a.ncols, bn64);
      a.use_patch = 0;
      a.accumulate = 0;
      configure_ksplit(a, src.out_elems, bm64, bn64, 8);  // the same rule on this tile's grid (chunks are 16 k rows here too)
      a.simple_epilogue = src.simple_epilogue && 8 * (int64_t)src.out_elems <= ((int64_t)1 << 30);
      k = psrc;
      k.KP = a.KP;
      k.MP = a.MP;
      k.kperm_T = 0;
      k.koff_invalid = 0;
      const int64_t pack_elems = (int64_t)a.G * a.KP * a.MP;
      if (pack_elems >= max64 || (int64_t)a.G * a.m_tiles * a.col_tiles >= ((int64_t)1 << 31)) d->f64_ok = 0;
      ws = (size_t)pack_elems * 8 + (size_t)a.KP * sizeof(KTabEntry) +
           (a.ksplit > 1 ? (size_t)a.ksplit * (size_t)src.out_elems * 8 : 0);
    };
    corr64(d->fwd, d->fwd_pack, d->fwd64, d->fwd64_pack, x_elems, d->fwd64_ws, d->fwd64_rows);
    corr64(d->bwd, d->bwd_pack, d->bwd64, d->bwd64_pack, y_elems, d->bwd64_ws, d->bwd64_rows);
    const int32_t bm64 = d->wg64_rows = f64_pick_rows(Kg, true);
    WgradArgs& a = d->wg64;
    a = d->wg;
    a.dy_bytes = (uint32_t)(8 * y_elems);
    a.x_bytes = (uint32_t)(8 * x_elems);
    a.bounds_mode = 1;
    a.m_tiles = (int32_t)ceil_div(Kg, bm64);
    a.n_tiles = (int32_t)ceil_div(kred, bn64);
    const int64_t tiles = G * a.m_tiles * a.n_tiles;
    int64_t S = 1024 / tiles;
    const int64_t max_by_len = ceil_div((int64_t)a.ncols, 4 * bk64);
    const int64_t max_by_ws = ((int64_t)8 << 20) / (w_elems > 0 ? w_elems : 1);
    if (S > max_by_len) S = max_by_len;
    if (S > max_by_ws) S = max_by_ws;
    if (S > 256) S = 256;
    if (S < 1) S = 1;
    a.cols_per_split = (int32_t)round_up(ceil_div((int64_t)a.ncols > 0 ? a.ncols : 1, S), bk64);
    a.S = (int32_t)ceil_div((int64_t)a.ncols > 0 ? a.ncols : 1, a.cols_per_split);
    if (a.S * w_elems >= max64 || tiles * a.S >= ((int64_t)1 << 31)) d->f64_ok = 0;
    d->wg64_ws = (size_t)a.S * (size_t)w_elems * 8;
    d->bg64_ws = 2 * d->bg_ws;
    auto e64 = [](const CorrArgs& c) { return c.simple_epilogue ? 's' : 'p'; };
    snprintf(d->names64, sizeof(d->names64),
             "fwd=corr64_%dx64x16[e%c](S=%d,L=%d);bwd_data=corr64_%dx64x16[e%c](S=%d,L=%d);"
             "bwd_filter=wgrad64_%dx64x16(S=%d,L=2);bwd_bias=bias_grad64(S=%d,L=2)",
             d->fwd64_rows, e64(d->fwd64), d->fwd64.ksplit, 2 + (d->fwd64.ksplit > 1), d->bwd64_rows, e64(d->bwd64),
             d->bwd64.ksplit, 2 + (d->bwd64.ksplit > 1) + (d->bwd_zero_fill != 0), d->wg64_rows, a.S,
             d->bg.S);
    d->ws_bytes64 = d->fwd64_ws;
    if (d->bwd64_ws > d->ws_bytes64) d->ws_bytes64 = d->bwd64_ws;
    if (d->wg64_ws > d->ws_bytes64) d->ws_bytes64 = d->wg64_ws;
    if (d->bg64_ws > d->ws_bytes64) d->ws_bytes64 = d->bg64_ws;
  }

  // ---- thin groups: direct kernels instead of the GEMM tiles ----
  {
    const int64_t taps = (int64_t)p.kernel_h * p.kernel_w;
    d->use_direct = G > 1 && taps <= 64 && direct_is_faster(Cg, Kg, p.kernel_h, p.kernel_w);
    DirectArgs& a = d->dir;
    a.bias_part = nullptr;
    a.N = p.n;
    a.C = p.c;
    a.H = p.h;
    a.W = p.w;
    a.K = p.num_output;
    a.OH = (int32_t)OH;
    a.OW = (int32_t)OW;
    a.kh = p.kernel_h;
    a.kw = p.kernel_w;
    a.sh = p.stride_h;
    a.sw = p.stride_w;
    a.ph = p.pad_h;
    a.pw = p.pad_w;
    a.dh = p.dilation_h;
    a.dw = p.dilation_w;
    a.Cg = (int32_t)Cg;
    a.Kg = (int32_t)Kg;
    a.x_elems = (uint32_t)x_elems;
    a.y_elems = (uint32_t)y_elems;
    a.w_elems = (uint32_t)w_elems;
    a.mOW = make_magic((uint32_t)OW);
    a.mOH = make_magic((uint32_t)OH);
    a.mK = make_magic((uint32_t)K);
    a.mKg = make_magic((uint32_t)Kg);
    a.mW = make_magic((uint32_t)W);
    a.mH = make_magic((uint32_t)H);
    a.mC = make_magic((uint32_t)C);
    a.mCg = make_magic((uint32_t)Cg);
    a.mSh = make_magic((uint32_t)p.stride_h);
    a.mSw = make_magic((uint32_t)p.stride_w);
    if (d->use_direct) {
      a.taps = (int32_t)taps;
      a.slots = (int32_t)(64 / taps);
      a.chunks_per_img = (int32_t)ceil_div(OH * OW, a.slots);
      a.mTaps = make_magic((uint32_t)taps);
      a.mKw = make_magic((uint32_t)p.kernel_w);
      a.mChunks = make_magic((uint32_t)a.chunks_per_img);
      // splits over the images: about a thousand workgroups, partial sums of at most 32 MiB
      int64_t S = ceil_div(1024, K * Cg);
      const int64_t max_by_ws = ((int64_t)8 << 20) / (w_elems > 0 ? w_elems : 1);
      if (S > max_by_ws) S = max_by_ws;
      if (S > N) S = N;
      if (S > 256) S = 256;
      if (S < 1) S = 1;
      a.imgs_per_split = (int32_t)ceil_div(N > 0 ? N : 1, S);
      a.S = (int32_t)ceil_div(N > 0 ? N : 1, a.imgs_per_split);
      if ((int64_t)N * a.chunks_per_img >= ((int64_t)1 << 31) || K * Cg >= ((int64_t)1 << 31) ||
          a.S * (w_elems + K) >= kMaxElems)
        d->use_direct = 0;
    }
    if (d->use_direct) {
      d->fwd_ws = d->bwd_ws = 0;
      d->wg_ws = (size_t)a.S * (size_t)w_elems * 4;
      d->wgb_ws = (size_t)a.S * (size_t)(w_elems + K) * 4;  // S x K sums of dy behind the filter partials
      d->fwd64_ws = d->bwd64_ws = 0;
      d->wg64_ws = 2 * d->wg_ws;
      d->ws_bytes64 = d->wg64_ws > d->bg64_ws ? d->wg64_ws : d->bg64_ws;
      char df[3][32];
      for (int pass = 0; pass < 3; ++pass) direct_form_name(pass, a, df[pass], sizeof(df[pass]));
      snprintf(d->names64, sizeof(d->names64),
               "fwd=direct64[%s](S=1,L=1);bwd_data=direct64[%s](S=1,L=1);bwd_filter=direct64[%s](S=%d,L=2);"
               "bwd_bias=bias_grad64(S=%d,L=2)",
               df[0], df[1], df[2], a.S, d->bg.S);
    }
  }

  d->ws_bytes = d->fwd_ws;
  if (d->bwd_ws > d->ws_bytes) d->ws_bytes = d->bwd_ws;
  if (d->wg_ws > d->ws_bytes) d->ws_bytes = d->wg_ws;
  if (d->bg_ws > d->ws_bytes) d->ws_bytes = d->bg_ws;
  if (p.bias_term && d->wgb_ws > d->ws_bytes) d->ws_bytes = d->wgb_ws;
  {
    // every template parameter and run-time branch that selects different kernel code is spelled out:
    // tile, bounds mode (m0/m1/m2) or patch staging, epilogue form (es/er/ep: separable offsets, range-
    // checked stores with compares, plain pointers), staging of the filter gradient (lds/reg), one or
    // two launches of the bias gradient
    char f[64], b[64], wg[64];
    corr_variant_name(f, sizeof(f), d->fwd_tile, d->fwd, 0, d->fwd_thin);
    corr_variant_name(b, sizeof(b), d->bwd_tile, d->bwd, d->bwd_zero_fill, d->bwd_thin);
    snprintf(wg, sizeof(wg), "%s[m%d,%s,e%c](S=%d,L=2)", wgrad_tile_name(d->wg_tile), d->wg.bounds_mode,
             d->wg_tile == WGRAD_128x128 ? "lds" : "reg", 4 * Kg * kred <= ((int64_t)1 << 30) ? 'r' : 'p', d->wg.S);
    if (d->use_direct) {
      char df[3][32];
      for (int pass = 0; pass < 3; ++pass) direct_form_name(pass, d->dir, df[pass], sizeof(df[pass]));
      snprintf(f, sizeof(f), "direct[%s](S=1,L=1)", df[0]);
      snprintf(b, sizeof(b), "direct[%s](S=1,L=1)", df[1]);
      snprintf(wg, sizeof(wg), "direct[%s](S=%d,L=2)", df[2], d->dir.S);
    }
    snprintf(d->names, sizeof(d->names), "fwd=%s;bwd_data=%s;bwd_filter=%s;bwd_bias=bias_grad[%s](S=%d,L=%d)", f, b, wg,
             d->bg_direct ? "one" : "two", d->bg.S, d->bg_direct ? 1 : 2);
  }
  *out = d;
  return CONV_OK;
}

int conv_desc_destroy(conv_desc_t* d) {
  if (!d) return CONV_EINVAL;
  delete d;
  return CONV_OK;
}

int conv_desc_output_shape(const conv_desc_t* d, int32_t* n, int32_t* k, int32_t* oh, int32_t* ow) {
  if (!d) return CONV_EINVAL;
  if (n) *n = d->p.n;
  if (k) *k = d->p.num_output;
  if (oh) *oh = d->OH;
  if (ow) *ow = d->OW;
  return CONV_OK;
}

int conv_desc_workspace_bytes(const conv_desc_t* d, size_t* bytes) {
  if (!d || !bytes) return CONV_EINVAL;
  *bytes = d->ws_bytes;
  return CONV_OK;
}

const char* conv_desc_kernel_names(const conv_desc_t* d) { return d ? d->names : ""; }

int conv_forward(const conv_desc_t* d, const float* x, const float* w, const float* bias, float* y, void* ws,
                 size_t ws_bytes, void* hip_stream) {
  return run_forward(d, x, w, bias, y, ws, ws_bytes, hip_stream);
}

int conv_backward_data(const conv_desc_t* d, const float* w, const float* dy, float* dx, void* ws, size_t ws_bytes,
                       void* hip_stream) {
  return run_backward_data(d, w, dy, dx, 0.f, ws, ws_bytes, hip_stream);
}

int conv_backward_filter(const conv_desc_t* d, const float* x, const float* dy, float* dw, float beta, void* ws,
                         size_t ws_bytes, void* hip_stream) {
  return run_backward_filter(d, x, dy, dw, beta, ws, ws_bytes, hip_stream, ReduceExtras());
}

int conv_backward_filter_bias(const conv_desc_t* d, const float* x, const float* dy, float* dw, float* db, float beta,
                              void* ws, size_t ws_bytes, void* hip_stream) {
  if (!d || !db) return CONV_EINVAL;
  if (!d->p.bias_term) return CONV_EINVAL;
  return run_backward_filter(d, x, dy, dw, beta, ws, ws_bytes, hip_stream, ReduceExtras(), db);
}

int conv_backward_bias(const conv_desc_t* d, const float* dy, float* db, float beta, void* ws, size_t ws_bytes,
                       void* hip_stream) {
  if (!d || !db) return CONV_EINVAL;
  if (!d->p.bias_term) return CONV_EINVAL;
  if (!(beta == 0.f || beta == 1.f)) return CONV_EINVAL;
  const bool empty = d->p.n == 0;
  if (!empty && !dy) return CONV_EINVAL;
  if (!empty && (!ws || ws_bytes < d->bg_ws)) return CONV_EWORKSPACE;
  BiasGradArgs a = d->bg;
  a.dy = dy;
  a.part = static_cast<float*>(ws);
  if (!empty && d->bg_direct) {  // small blob: one launch writes db
    a.db = db;
    a.beta = beta;
    const int e1 = launch_bias_grad(a, hip_stream);
    return e1 ? record_hip_error(e1) : CONV_OK;
  }
  int e = empty ? 0 : launch_bias_grad(a, hip_stream);
  if (e) return record_hip_error(e);
  ReduceArgs r = {};
  r.part = a.part;
  r.dst = db;
  r.count = d->p.num_output;
  r.S = empty ? 0 : a.S;
  r.beta = beta;
  e = launch_reduce(r, hip_stream);
  return e ? record_hip_error(e) : CONV_OK;
}

// ---- double base type ----

const char* conv_desc_kernel_names_f64(const conv_desc_t* d) { return d && d->f64_ok ? d->names64 : ""; }

int conv_desc_workspace_bytes_f64(const conv_desc_t* d, size_t* bytes) {
  if (!d || !bytes) return CONV_EINVAL;
  if (!d->f64_ok) return CONV_ESHAPE;
  *bytes = d->ws_bytes64;
  return CONV_OK;
}

static int run_corr64(const conv_desc_t* d, int32_t tile_rows, const CorrArgs& args, const PackArgs& pack, size_t need,
                      const double* w, const double* in, const double* bias, double* out, size_t zero_out_bytes,
                      void* ws, size_t ws_bytes, void* hip_stream) {
  if (!d->f64_ok) return CONV_ESHAPE;
  if (!ws || ws_bytes < need) return CONV_EWORKSPACE;
  PackArgs k = pack;
  const size_t pack_bytes = (size_t)k.G * k.KP * k.MP * 8 + (size_t)k.KP * sizeof(KTabEntry);
  double* const part = reinterpret_cast<double*>(static_cast<char*>(ws) + pack_bytes);
  if (zero_out_bytes) {  // backward data with row / column phases no tap reaches: clear dx, or the slices' partial sums
    const int ez = args.ksplit > 1 ? launch_fill_zero(part, (size_t)args.ksplit * zero_out_bytes, hip_stream)
                                   : launch_fill_zero(out, zero_out_bytes, hip_stream);
    if (ez) return record_hip_error(ez);
  }
  k.w = reinterpret_cast<const float*>(w);
  k.A = static_cast<float*>(ws);
  k.ktab = reinterpret_cast<KTabEntry*>(static_cast<double*>(ws) + (size_t)k.G * k.KP * k.MP);
  int e = launch_pack(k, hip_stream, true);
  if (e) return record_hip_error(e);
  CorrArgs a = args;
  a.A = k.A;
  a.ktab = k.ktab;
  a.in = reinterpret_cast<const float*>(in);
  a.bias = reinterpret_cast<const float*>(bias);
  a.out = reinterpret_cast<float*>(out);
  a.part = reinterpret_cast<float*>(part);
  e = launch_corr64(tile_rows, a, hip_stream);
  if (e) return record_hip_error(e);
  if (a.ksplit > 1) {  // add the slices and the bias
    ReduceArgs r = {};
    r.part = a.part;
    r.dst = a.out;
    r.count = a.out_elems;
    r.S = a.ksplit;
    r.beta = 0.f;
    r.bias = a.bias;
    r.chan_elems = d->OH * d->OW;
    r.channels = d->p.num_output;
    r.mChanElems = make_magic(r.chan_elems);
    r.mChannels = make_magic(r.channels);
    e = launch_reduce64(r, hip_stream);
  }
  return e ? record_hip_error(e) : CONV_OK;
}

int conv_forward_f64(const conv_desc_t* d, const double* x, const double* w, const double* bias, double* y, void* ws,
                     size_t ws_bytes, void* hip_stream) {
  if (!d || !w) return CONV_EINVAL;
  if ((d->p.bias_term != 0) != (bias != nullptr)) return CONV_EINVAL;
  if (d->p.n == 0) return CONV_OK;
  if (!x || !y) return CONV_EINVAL;
  if (d->use_direct && d->f64_ok) {
    DirectArgs da = d->dir;
    da.in = x;
    da.w = w;
    da.bias = bias;
    da.out = y;
    const int ed = launch_direct(0, da, true, hip_stream);
    return ed ? record_hip_error(ed) : CONV_OK;
  }
  return run_corr64(d, d->fwd64_rows, d->fwd64, d->fwd64_pack, d->fwd64_ws, w, x, bias, y, 0, ws, ws_bytes,
                    hip_stream);
}

int conv_backward_data_f64(const conv_desc_t* d, const double* w, const double* dy, double* dx, void* ws,
                           size_t ws_bytes, void* hip_stream) {
  if (!d || !w) return CONV_EINVAL;
  if (d->p.n == 0) return CONV_OK;
  if (!dy || !dx) return CONV_EINVAL;
  if (d->use_direct && d->f64_ok) {
    DirectArgs da = d->dir;
    da.in = dy;
    da.w = w;
    da.out = dx;
    const int ed = launch_direct(1, da, true, hip_stream);
    return ed ? record_hip_error(ed) : CONV_OK;
  }
  const size_t zero = d->bwd_zero_fill ? (size_t)d->bwd64.out_elems * 8 : 0;
  return run_corr64(d, d->bwd64_rows, d->bwd64, d->bwd64_pack, d->bwd64_ws, w, dy, nullptr, dx, zero, ws, ws_bytes,
                    hip_stream);
}

int conv_backward_filter_f64(const conv_desc_t* d, const double* x, const double* dy, double* dw, double beta,
                             void* ws, size_t ws_bytes, void* hip_stream) {
  if (!d || !dw) return CONV_EINVAL;
  if (!(beta == 0.0 || beta == 1.0)) return CONV_EINVAL;
  if (!d->f64_ok) return CONV_ESHAPE;
  const bool empty = d->p.n == 0;
  if (!empty && (!x || !dy)) return CONV_EINVAL;
  if (!empty && (!ws || ws_bytes < d->wg64_ws)) return CONV_EWORKSPACE;
  WgradArgs a = d->wg64;
  a.dy = reinterpret_cast<const float*>(dy);
  a.x = reinterpret_cast<const float*>(x);
  a.part = static_cast<float*>(ws);
  int e = 0;
  if (d->use_direct) {
    DirectArgs da = d->dir;
    da.in = x;
    da.w = dy;
    da.part = ws;
    a.S = da.S;
    if (!empty) e = launch_direct(2, da, true, hip_stream);
  } else if (!empty) {
    e = launch_wgrad64(d->wg64_rows, a, hip_stream);
  }
  if (e) return record_hip_error(e);
  ReduceArgs r = {};
  r.part = a.part;
  r.dst = reinterpret_cast<float*>(dw);
  r.count = (int32_t)((int64_t)d->p.num_output * d->wg64.Kred);
  r.S = empty ? 0 : a.S;
  r.beta = (float)beta;
  e = launch_reduce64(r, hip_stream);
  return e ? record_hip_error(e) : CONV_OK;
}

int conv_backward_bias_f64(const conv_desc_t* d, const double* dy, double* db, double beta, void* ws, size_t ws_bytes,
                           void* hip_stream) {
  if (!d || !db) return CONV_EINVAL;
  if (!d->p.bias_term) return CONV_EINVAL;
  if (!(beta == 0.0 || beta == 1.0)) return CONV_EINVAL;
  if (!d->f64_ok) return CONV_ESHAPE;
  const bool empty = d->p.n == 0;
  if (!empty && !dy) return CONV_EINVAL;
  if (!empty && (!ws || ws_bytes < d->bg64_ws)) return CONV_EWORKSPACE;
  BiasGradArgs a = d->bg;
  a.dy = reinterpret_cast<const float*>(dy);
  a.part = static_cast<float*>(ws);
  int e = empty ? 0 : launch_bias_grad64(a, hip_stream);
  if (e) return record_hip_error(e);
  ReduceArgs r = {};
  r.part = a.part;
  r.dst = reinterpret_cast<float*>(db);
  r.count = d->p.num_output;
  r.S = empty ? 0 : a.S;
  r.beta = (float)beta;
  e = launch_reduce64(r, hip_stream);
  return e ? record_hip_error(e) : CONV_OK;
}

const char* conv_status_string(int status) {
  switch (status) {
    case CONV_OK: return "success";
    case CONV_EINVAL: return "invalid argument";
    case CONV_ESHAPE: return "unsupported shape (empty output or a tensor too large for 32-bit offsets)";
    case CONV_EWORKSPACE: return "workspace missing or too small";
    case CONV_EHIP: return "HIP launch failed";
    default: return "unknown status";
  }
}

int conv_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
