// Internal declarations shared by the host-side descriptor code and the gfx950 kernels.
// Nothing here is part of the public boundary (that is include/mi355conv.h).
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "mi355conv.h"

namespace mi355conv {

// Unsigned division by a run-time constant with one multiply-high, one add and one shift
// (Granlund-Montgomery round-up method).  Exact for dividends below 2^31.
struct Magic {
  uint32_t mul;
  uint32_t shift;
};

inline Magic make_magic(uint32_t d) {
  Magic m;
  uint32_t s = 0;
  while ((1ull << s) < d) ++s;
  m.shift = s;
  m.mul = (uint32_t)(((1ull << 32) * ((1ull << s) - d)) / d + 1);
  return m;
}

// ---------------------------------------------------------------------------------------------
// "Correlation" kernels: forward and backward-data share one implicit-GEMM kernel
//   D[m][col] = sum_kk A[kk][m] * gather(in)[kk][col]
// with kk = (channel, tap_h, tap_w), col = (image, a, b), and a table-driven epilogue that
// scatters row m / column col to its place in the output blob.
// Per reduction index kk = (c, i, j): byte offset c*IH*IW + i*dh*IW + j*dw of the tap and its
// row / column displacement (for the bounds test).  Entries past the reduction length carry a
// row displacement that fails every bounds test.
struct KTabEntry {
  uint32_t koff;
  int32_t idh, jdw;
  int32_t tap;  // i*TW + j (mod 32): bit index into a column's tap bitmask
};

constexpr int kMaxPhases = 8;  // phase tables of the backward-data row space (larger sets stay dense)

struct CorrArgs {
  const float* A;     // packed operand, [G][MP][KP] floats, zero padded
  const KTabEntry* ktab;  // [KP], written by the pack kernel
  const float* in;    // blob that is gathered, [N][in_chan_total][IH][IW]
  const float* bias;  // per output channel, or null
  float* out;
  uint32_t in_bytes;  // size of `in`, the range of the gather's hardware bounds check
  int32_t bounds_mode;  // 0 no padding, 1 compares, 2 tap bitmask (see corr_kernel)
  // column space
  int32_t ncols, P, PW;  // ncols = N*P, P = PH*PW
  Magic mP, mPW;
  // gather geometry: row = a*sh - ph + i*dh, column = b*sw - pw + j*dw
  int32_t IH, IW, IHW;
  int32_t in_img_stride;  // elements between images of `in`
  int32_t in_grp_stride;  // elements between the channel blocks of two groups
  int32_t TW, THW;        // taps per row, taps per channel
  Magic mTW, mTHW;
  int32_t sh, sw, dh, dw, ph, pw;
  int32_t Kred, KP;   // reduction length and its padded size (multiple of the k tile)
  int32_t Mrows, MP;  // rows per group and padded rows (multiple of the m tile)
  // epilogue: row m = (c*RSh + ph)*RSw + pw lands at channel g*chan_per_grp + c, spatial
  // (a*OSh + rh - opad_h, b*OSw + rw - opad_w) of an [N][*][OHd][OWd] blob, where rh = ph, or
  // phase_h[ph] when tab_h is set (backward data keeps only the row phases that some tap reaches:
  // RSh of the OSh phases; the same for columns).  Forward: everything 1.
  int32_t RSw, RShw;
  Magic mRSw, mRShw;
  int32_t RSh;
  int32_t OSh, OSw;
  int32_t tab_h, tab_w;
  int32_t phase_h[kMaxPhases], phase_w[kMaxPhases];
  int32_t opad_h, opad_w;
  int32_t OHd, OWd;
  int32_t out_img_stride;
  int32_t chan_per_grp;
  // grid
  int32_t G, m_tiles, col_tiles;
  // split reduction (small problems): ksplit slices of chunks_per_split k chunks each write partial
  // outputs to part[split][out_elems]; a reduce kernel finishes.  ksplit = 1: none of this.
  int32_t ksplit, chunks_per_split;
  int32_t out_elems;
  float* part;
  // add to what the output already holds instead of overwriting it (unsplit launches only; a
  // split launch accumulates in its reduce kernel)
  int32_t accumulate;
  // patch-staged variant (corr_patch_kernel); use_patch = 0 selects the gather kernel
  int32_t use_patch;
  int32_t Cg_in;       // gathered channels per group (multiple of 8)
  int32_t NS;          // super steps = Cg_in/8 * taps
  int32_t PH;          // rows of the column space per image (P / PW)
  int32_t Nimg;        // images
  int32_t PWID, PSZ;   // patch row length (PW + TW - 1); floats per channel of an LDS patch stage
  Magic mPWID, mRSEG;  // divisions by PWID and by the patch rows of a full image (PH + TH - 1)
  int32_t simple_epilogue;  // one phase per channel and an output of at most 2^30 bytes: offset-only epilogue
  // LDS-staged form of corr_thin_kernel: A is the weight blob itself (no pack kernel); element strides of
  // a GEMM row, a gathered channel and a group in it, and whether the taps run backwards (backward data)
  int32_t w_row_stride, w_chan_stride, w_grp_stride, w_reversed;
};

constexpr int kPatchEPT = 3;  // patch elements per thread and channel: PSZ <= 3 * 256

// Packs the weights into the A operand of the correlation kernel.
//   mode 0 (forward): A[g][m][kk] = w[g*Kg + m][kk]
//   mode 1 (backward data): rows m = (c, rh, rw), kk = (k, qh', qw'); the entry is
//     w[g*Kg + k][c][i][j] with i*dil_h = stride_h*eh*(Qh-1-qh') + rh (and likewise j), else 0.
struct PackArgs {
  const float* w;
  float* A;
  KTabEntry* ktab;
  int32_t tTW, tTHW, tIW, tIHW, tdh, tdw;  // gather geometry for the k table
  uint32_t koff_invalid;                   // offset of k rows past the reduction length
  int32_t mode;
  int32_t G, Kg, Cg, kh, kw;
  int32_t sh, sw, dh, dw;
  int32_t Qh, Qw;
  // backward data: nvh x nvw row phases per channel (phase value = index, or phase_h[index] when
  // tab_h is set); tap slot q of a phase sits q*eh rows of dy away
  int32_t nvh, nvw, eh, ew;
  int32_t tab_h, tab_w;
  int32_t phase_h[kMaxPhases], phase_w[kMaxPhases];
  int32_t Kred, KP, Mrows, MP;
  int32_t kperm_T;  // 0, or the tap count T: k runs (8-channel chunk, tap, channel in chunk) instead of (c, tap)
};

// Backward filter: part[s][g][k][nn] = sum over the split's columns of dy * gathered x.
struct WgradArgs {
  const float* dy;
  const float* x;
  float* part;
  uint32_t dy_bytes, x_bytes;  // sizes of the two blobs: the ranges of the hardware bounds checks
  int32_t bounds_mode;         // 0 no padding, 1 compares, 2 tap bitmask (see wgrad_kernel)
  int32_t ncols, P, PW;
  Magic mP, mPW;
  int32_t Kg, Ktot;
  int32_t Cg, C, H, W, HW;
  int32_t kw, khw;
  Magic mKW, mKHW;
  int32_t sh, sw, dh, dw, ph, pw;
  int32_t Kred;
  int32_t cols_per_split, S;
  int32_t G, m_tiles, n_tiles;
  // Elements between the partial slices of two splits (G*Kg*Kred).
  int32_t part_stride;
  // Bias gradient riding along (null: not wanted): the row sums of dy.  Every workgroup adds up the dy
  // tiles of the chunks ch with ch % n_tiles == its n_tile, so the work is spread over all column
  // tiles: bias_part[(s*n_tiles + n_tile)*Ktot + g*Kg + k] = that share of the sum of
  // dy[., g*Kg + k, .] over the split's columns.
  float* bias_part;
};

struct ReduceArgs {
  const float* part;  // [S][stride]: elements [0, count) of a slice go to dst
  float* dst;         // [count]
  int32_t count, S;
  int32_t stride;     // elements between slices (0: count)
  // second reduction of the same launch with the same beta (filter + bias gradient together):
  // dst2[count2] from part2[S2][count2]; the workgroups past the first reduction's take it
  const float* part2;
  float* dst2;
  int32_t count2, S2;
  float beta;
  // optional per-channel bias for blobs laid out [..][channel][chan_elems]: dst += bias[(i / chan_elems) % channels]
  const float* bias;
  int32_t chan_elems, channels;
  Magic mChanElems, mChannels;
  int32_t relu;  // clamp the finished value at zero from below
};

// Element-wise and column-sum helpers of the InnerProduct layer.
struct ReluBwdArgs {
  const float* y;   // [count] output of the forward pass
  const float* dy;  // [count]
  float* dz;        // [count] = y > 0 ? dy : 0   (may alias dy)
  int32_t count;
};

struct ColSumArgs {
  const float* src;  // [rows][cols]
  float* part;       // [S][cols]
  int32_t rows, cols, S, rows_per_split;
  // small matrices: one launch finishes dst = beta*dst + column sums (dst null otherwise)
  float* dst;
  float beta;
};

struct BiasGradArgs {
  const float* dy;  // [N][K][P]
  float* part;      // [K][S]
  int32_t N, K, P;
  int32_t S;        // splits over the images
  int32_t n_per_split;
  // S == 1 on a small blob: the kernel finishes db itself (db = beta*db + sum) and no reduce
  // kernel follows; db is null otherwise
  float* db;
  float beta;
};

// Direct (no matrix unit) kernels for thin groups -- depthwise convolution and its neighbours,
// where a group's GEMM has one to a few rows and a handful of reduction indices and the MFMA tiles
// would be almost all padding.  The pointer members address floats or doubles.
struct DirectArgs {
  const void* in;    // forward, filter gradient: x; backward data: dy
  const void* w;     // forward, backward data: weights; filter gradient: dy
  const void* bias;  // forward only (may be null)
  void* out;         // y / dx
  void* part;        // filter gradient: [S][K][Cg][kh][kw] partial sums
  void* bias_part;   // filter gradient: when not null, [S][K] sums of dy (the workgroups of input channel 0 of a
                     // group add up the dy values they read: the bias gradient from the same pass)
  int32_t N, C, H, W, K, OH, OW, kh, kw, sh, sw, ph, pw, dh, dw, Cg, Kg;
  uint32_t x_elems, y_elems, w_elems;
  Magic mOW, mOH, mK, mKg;             // forward: output index -> (n, k, oh, ow), k -> group
  Magic mW, mH, mC, mCg, mSh, mSw;     // backward data: input index -> (n, c, h, w), divisions by the stride
  // filter gradient: lanes = (position slot, tap); a workgroup = one (k, c) pair x one run of images
  int32_t taps, slots;                 // kh*kw <= 64; slots = 64 / taps positions per wave and iteration
  int32_t chunks_per_img;              // ceil(OH*OW / slots)
  int32_t S, imgs_per_split;
  Magic mTaps, mKw, mChunks;
  // 3x3 and 5x5 kernels: a thread takes R consecutive output rows of one column (R = 8 or 4)
  int32_t OHB;                         // ceil(OH / R)
  Magic mOHB;
  int32_t OWQ;                         // four columns per thread: OW / 4
  Magic mOWQ;
  uint32_t row_items;                  // N*K*OHB*OW
  uint32_t w_out_stride, w_in_stride;  // weight index = group block + out*w_out_stride + in*w_in_stride + tap
  // 3x3 and 5x5 backward data at stride 2: a thread takes one stride x stride block of dx
  int32_t BH, BW;                      // blocks per image: ceil((H + ph) / stride), ceil((W + pw) / stride)
  Magic mBH, mBW;
  uint32_t block_items;                // N*C*BH*BW
};

// Tile variants, chosen once per descriptor.
enum CorrTile : int32_t {
  CORR_128x128 = 0,  // 32x32x2 MFMA, 2x2 waves of 64x64
  CORR_128x64,       // 32x32x2, 2x2 waves of 64x32
  CORR_96x128,       // 32x32x2, 1x4 waves of 96x32
  CORR_64x128,       // 32x32x2, 1x4 waves of 64x32
  CORR_64x64,        // 32x32x2, 2x2 waves of 32x32
  CORR_32x256,       // 32x32x2, 1x4 waves of 32x64
  CORR_32x128,       // 32x32x2, 1x4 waves of 32x32
  CORR_48x256,       // 16x16x4, 1x4 waves of 48x64
  CORR_48x128,       // 16x16x4, 1x4 waves of 48x32
  CORR_16x256,       // 16x16x4, 1x4 waves of 16x64
  CORR_16x64,        // 16x16x4, 1x4 waves of 16x16
  CORR_TILE_COUNT
};
enum WgradTile : int32_t {
  WGRAD_128x128 = 0,  // 2x2 waves of 64x64
  WGRAD_96x128,       // 1x4 waves of 96x32
  WGRAD_64x128,       // 1x4 waves of 64x32
  WGRAD_32x128,       // 1x4 waves of 32x32
  WGRAD_128x64,       // 2x2 waves of 64x32
  WGRAD_TILE_COUNT
};

void corr_tile_shape(int32_t tile, int32_t* bm, int32_t* bn, int32_t* bk);
void wgrad_tile_shape(int32_t tile, int32_t* bm, int32_t* bn, int32_t* bk);
const char* corr_tile_name(int32_t tile);
const char* wgrad_tile_name(int32_t tile);

// Launchers (defined next to the kernels).  Each returns the hipError_t of the launch as int.
int launch_pack(const PackArgs& a, void* stream, bool f64 = false);
int launch_corr(int32_t tile, const CorrArgs& a, void* stream);
int launch_corr_patch(int32_t tile, const CorrArgs& a, void* stream);
int launch_corr_thin(const CorrArgs& a, void* stream);  // Mrows <= 4, offset-only epilogue, no split
int launch_wgrad(int32_t tile, const WgradArgs& a, void* stream);
int launch_reduce(const ReduceArgs& a, void* stream);
int launch_bias_grad(const BiasGradArgs& a, void* stream);
int launch_fill_zero(void* dst, size_t bytes, void* stream);  // bytes a multiple of 4
// pass: 0 forward, 1 backward data (dx overwritten), 2 filter-gradient partials
int launch_direct(int pass, const DirectArgs& a, bool f64, void* stream);
// The kernel form launch_direct takes for a pass (decided from the parameters and the alignment of
// the pointers in `a`; null pointers count as aligned) and its name for conv_desc_kernel_names.
enum DirectFormKind : int32_t {
  DF_ELEM = 0,     // one output (or dx) element per thread, any kernel size
  DF_ELEM_K3,      // the same with the 3x3 taps unrolled
  DF_ROWS,         // 3x3 / 5x5: a thread owns 8 (unit stride and dilation) or 4 rows of one column
  DF_ROWS_VEC,     // 3x3 / 5x5 "same" layers: 4 rows x 4 columns per thread, 16-byte accesses
  DF_S2,           // 3x3 / 5x5 at stride 2: 4 rows x 2 output columns per thread
  DF_BWD_S2_VEC,   // backward data at stride 2: 2 rows x 4 columns of dx per thread
  DF_BWD_BLOCKS,   // backward data at stride 2: one 2x2 block of dx per thread
  DF_WGRAD_TAPS    // filter gradient, any kernel size: lanes = (position slot, tap)
};
struct DirectForm {
  DirectFormKind kind;
  bool unit;  // unit stride and dilation
};
DirectForm direct_form(int pass, const DirectArgs& a, size_t elem_bytes);
void direct_form_name(int pass, const DirectArgs& a, char* buf, size_t len);
// double base type: the same argument structs, pointer members addressing doubles
constexpr int32_t kF64TileCols = 64, kF64TileK = 16;
int32_t f64_pick_rows(int64_t rows, bool filter_gradient);  // 96, 64, 48, 32 or 16: pads `rows` least
int launch_corr64(int32_t tile_rows, const CorrArgs& a, void* stream);
int launch_wgrad64(int32_t tile_rows, const WgradArgs& a, void* stream);
int launch_reduce64(const ReduceArgs& a, void* stream);
int launch_bias_grad64(const BiasGradArgs& a, void* stream);
int launch_relu_bwd(const ReluBwdArgs& a, void* stream);
int launch_colsum(const ColSumArgs& a, void* stream);

// What the reduce kernel of a pass adds on top of the plain sum (all optional).
struct ReduceExtras {
  const float* bias = nullptr;  // bias[(i / chan_elems) % channels]
  int32_t chan_elems = 1, channels = 1;
  int32_t relu = 0;
};

// The passes behind the C entry points, with the extra knobs the InnerProduct layer needs
// (it runs as the same three contractions with the operand roles exchanged).
int run_forward(const conv_desc* d, const float* x, const float* w, const float* bias, float* y, void* ws,
                size_t ws_bytes, void* stream);
int run_backward_data(const conv_desc* d, const float* w, const float* dy, float* dx, float beta, void* ws,
                      size_t ws_bytes, void* stream);
// db non-null: also db = beta*db + row sums of dy, from the same read of dy
int run_backward_filter(const conv_desc* d, const float* x, const float* dy, float* dw, float beta, void* ws,
                        size_t ws_bytes, void* stream, const ReduceExtras& extras, float* db = nullptr);
int record_hip_error(int e);  // remembers e for conv_last_hip_error and returns CONV_EHIP
// workspace bytes conv_backward_filter needs for this descriptor (at most its conv_desc_workspace_bytes)
int conv_desc_backward_filter_workspace_bytes(const conv_desc* d, size_t* bytes);

}  // namespace mi355conv

// The descriptor: everything that can be decided from the parameters alone.
struct conv_desc {
  conv_params_t p;
  int32_t OH, OW;
  int32_t Cg, Kg;
  // forward
  int32_t fwd_tile;
  int32_t fwd_thin, bwd_thin;  // the pass runs corr_thin_kernel (at most four GEMM rows per group)
  mi355conv::CorrArgs fwd;  // pointers left null
  mi355conv::PackArgs fwd_pack;
  size_t fwd_ws, fwd_pack_bytes;
  // backward data
  int32_t bwd_tile;
  mi355conv::CorrArgs bwd;
  mi355conv::PackArgs bwd_pack;
  size_t bwd_ws, bwd_pack_bytes;
  int32_t bwd_zero_fill;  // some row / column phases of dx are reached by no tap: zero dx first
  // backward filter
  int32_t wg_tile;
  mi355conv::WgradArgs wg;
  size_t wg_ws;
  size_t wgb_ws;  // filter and bias gradient together (conv_backward_filter_bias)
  // backward bias
  mi355conv::BiasGradArgs bg;
  size_t bg_ws;
  int32_t bg_direct;  // fp32: the bias-gradient kernel writes db itself (small blobs)
  size_t ws_bytes;
  // thin groups: all three passes run the direct kernels (both base types)
  int32_t use_direct;
  mi355conv::DirectArgs dir;
  char names[256];
  // double base type: tiles of fwd64_rows / bwd64_rows / wg64_rows x 64 x 16 (f64_ok = 0: a blob of
  // 2^29 or more elements)
  int32_t f64_ok;
  int32_t fwd64_rows, bwd64_rows, wg64_rows;
  char names64[256];
  mi355conv::CorrArgs fwd64, bwd64;
  mi355conv::PackArgs fwd64_pack, bwd64_pack;
  size_t fwd64_ws, bwd64_ws;
  mi355conv::WgradArgs wg64;
  size_t wg64_ws, bg64_ws, ws_bytes64;
};
