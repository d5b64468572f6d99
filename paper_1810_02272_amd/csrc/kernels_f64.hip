// Double-precision base type for the convolution layer (the paper builds every layer for either
// a float or a double base type, section after Table 1): the same four passes on the fp64 matrix
// instruction v_mfma_f64_16x16x4f64.  Workgroup tiles of 96/64/48/32/16 rows by 64 columns by 16 k
// (the row count that pads the matrix least is chosen per pass), MODE-1 style bounds checks (row
// and column compares, out-of-image elements read as 0 through the buffer range check), a
// two-stage LDS ring with a register prefetch.  The argument structs are those of the fp32
// kernels; their pointer members address doubles here and the byte counts are those of doubles.
//
// fp64 MFMA lane layout (one wave computes a 16x16 tile, 4 k values per instruction):
//   lane l feeds A[l%16][l/16] and B[l/16][l%16]; accumulator register r of lane l holds
//   D[4*r + l/16][l%16].
#include <hip/hip_runtime.h>

#include "device_utils.h"
#include "internal.h"

namespace mi355conv {

namespace {

typedef double f64x2 __attribute__((ext_vector_type(2)));
typedef double f64x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int BN = 64, BK = 16;
// LDS tiles are [k][row] with an odd row count per k (BM + 1, 65): an 8-byte operand read (lane ->
// row l%16, k 4s + l/16) takes 16 consecutive doubles per quarter wave, and a staging write whose
// lanes run along k (filter gradient) steps through the 32 banks two at a time.

// Four waves as WM x WN, each owning MB x NB MFMA tiles of 16x16: BM = WM*MB*16 rows, 64 columns.
template <int MB, int NB, int WM, int WN>
struct Cfg64 {
  static constexpr int BM = WM * MB * 16;
  static constexpr int LDA = BM + 1, LDB = BN + 1;      // doubles per k row of the two tiles
  static constexpr int STAGE = BK * (LDA + LDB);        // doubles per stage
  static constexpr int A_PER = (BM * 4 + kThreads - 1) / kThreads;  // 32-byte pieces of the A tile per thread
  static_assert(WM * WN == 4 && WN * NB * 16 == BN, "four waves, 64 columns");
};

__device__ __forceinline__ double buffer_load_f64(__amdgpu_buffer_rsrc_t rsrc, uint32_t off) {
  return __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(rsrc, off, 0, 0));
}

__device__ __forceinline__ void mfma64(double a, double b, f64x4& c) {
  c = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

// One chunk (BK k values) of a wave's MB x NB MFMA tiles.
template <int MB, int NB, int LDA, int LDB>
__device__ __forceinline__ void chunk_mfma(const double* sA, const double* sB, f64x4 (&acc)[MB][NB]) {
#pragma unroll
  for (int s = 0; s < BK / 4; ++s) {
    double av[MB], bv[NB];
#pragma unroll
    for (int i = 0; i < MB; ++i) av[i] = sA[4 * s * LDA + i * 16];
#pragma unroll
    for (int j = 0; j < NB; ++j) bv[j] = sB[4 * s * LDB + j * 16];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) mfma64(av[i], bv[j], acc[i][j]);
  }
}

// D[m][col] = sum_kk A[m][kk] * gather(in)[kk][col]: forward and backward data (see corr_kernel
// for the fp32 version and the meaning of every CorrArgs field).
template <int MB, int NB, int WM, int WN>
__global__ __launch_bounds__(kThreads) void corr64_kernel(const CorrArgs a) {
  using C = Cfg64<MB, NB, WM, WN>;
  constexpr int BM = C::BM, STAGE = C::STAGE, A_PER = C::A_PER, LDA = C::LDA, LDB = C::LDB;
  __shared__ __align__(16) double smem[2 * STAGE];
  const int t = threadIdx.x, lane = t & 63;
  const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wv / WN, wn = wv % WN;

  uint32_t lin = xcd_contiguous_block_id();
  const uint32_t m_tile = lin % (uint32_t)a.m_tiles;
  lin /= (uint32_t)a.m_tiles;
  const uint32_t col_tile = lin % (uint32_t)a.col_tiles;
  lin /= (uint32_t)a.col_tiles;
  const uint32_t g = lin % (uint32_t)a.G;
  const uint32_t split = lin / (uint32_t)a.G;  // slice of the reduction (usually the only one)
  const int kc_first = (int)split * a.chunks_per_split;

  // the column this lane gathers
  uint32_t cbase = 0;
  int cih0 = -(1 << 29), ciw0 = 0;
  {
    const uint32_t col = col_tile * BN + lane;
    if (col < (uint32_t)a.ncols) {
      const uint32_t n = mdiv(col, a.mP);
      const uint32_t pix = col - n * a.P;
      const uint32_t pa = mdiv(pix, a.mPW);
      const uint32_t pb = pix - pa * a.PW;
      cih0 = (int)pa * a.sh - a.ph;
      ciw0 = (int)pb * a.sw - a.pw;
      cbase = 8u * (uint32_t)((int)(n * a.in_img_stride + g * a.in_grp_stride) + cih0 * a.IW + ciw0);
    }
  }
  const double* Ag =
      reinterpret_cast<const double*>(a.A) + ((size_t)g * a.MP + (size_t)m_tile * BM) * a.KP + (size_t)kc_first * BK;
  const KTabEntry* const ktab = a.ktab + kc_first * BK;  // chunk indices below are relative to the slice
  // Piece p = t + 256*i of the A tile: k quad p / BM, row p % BM (consecutive lanes on consecutive
  // rows: the four 8-byte LDS writes of a piece are conflict free).
  const __amdgpu_buffer_rsrc_t in_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.in), 0, (int)a.in_bytes, 0x00020000);

  f64x4 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[i][j] = f64x4{0., 0., 0., 0.};

  // Two register sets (see the loop below): f64x2 pairs of the A tile, four gathered k rows.
  f64x2 raX[A_PER][2], raY[A_PER][2];
  double rbX[4], rbY[4];
  // k-table entries of this wave's four k rows (uniform over the wave: scalar loads), fetched one
  // iteration before the gather that uses them so that it never waits on scalar memory
  KTabEntry te[4], te_next[4];
  auto load_tab = [&](int kc) {
#pragma unroll
    for (int e = 0; e < 4; ++e) te_next[e] = ktab[kc * BK + wv * 4 + e];
  };
  auto swap_tab = [&]() {
#pragma unroll
    for (int e = 0; e < 4; ++e) te[e] = te_next[e];
  };
  auto load_chunk = [&](f64x2(&ra)[A_PER][2], double(&rb)[4], int kc) {
#pragma unroll
    for (int p = 0; p < A_PER; ++p) {
      const int piece = t + kThreads * p;
      if (piece < BM * 4) {
        const double* src = Ag + (size_t)(piece % BM) * a.KP + kc * BK + (piece / BM) * 4;
        ra[p][0] = *reinterpret_cast<const f64x2*>(src);
        ra[p][1] = *reinterpret_cast<const f64x2*>(src + 2);
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int ih = cih0 + te[e].idh, iw = ciw0 + te[e].jdw;
      const bool ok = ((uint32_t)ih < (uint32_t)a.IH) & ((uint32_t)iw < (uint32_t)a.IW);
      // the k table holds byte offsets of 4-byte elements
      rb[e] = buffer_load_f64(in_rsrc, ok ? cbase + 2u * te[e].koff : a.in_bytes);
    }
  };
  auto store_chunk = [&](f64x2(&ra)[A_PER][2], double(&rb)[4], int buf) {
#pragma unroll
    for (int p = 0; p < A_PER; ++p) {
      const int piece = t + kThreads * p;
      if (piece < BM * 4) {
        double* sa = smem + buf * STAGE + (piece / BM) * 4 * LDA + piece % BM;
        sa[0] = ra[p][0][0];
        sa[LDA] = ra[p][0][1];
        sa[2 * LDA] = ra[p][1][0];
        sa[3 * LDA] = ra[p][1][1];
      }
    }
    double* sb = smem + buf * STAGE + BK * LDA + wv * 4 * LDB + lane;
#pragma unroll
    for (int e = 0; e < 4; ++e) sb[e * LDB] = rb[e];
  };

  // Pipeline, three chunks deep: while chunk kc is multiplied out of one LDS buffer, the register
  // set holding chunk kc+1 (loaded two iterations ago) is written to the other buffer and reloaded
  // with chunk kc+3; the other set holds chunk kc+2.  Chunk indices past the end are clamped: the
  // last iterations re-load and re-store the final chunk into a buffer nobody reads.
  int nchunks = a.KP / BK - kc_first;
  if (nchunks > a.chunks_per_split) nchunks = a.chunks_per_split;
  const int last = nchunks - 1;
  const double* opA = smem + (lane >> 4) * LDA + wm * MB * 16 + (lane & 15);
  const double* opB = smem + BK * LDA + (lane >> 4) * LDB + wn * NB * 16 + (lane & 15);
  load_tab(0);
  swap_tab();
  load_chunk(raX, rbX, 0);
  store_chunk(raX, rbX, 0);
  load_tab(last < 1 ? last : 1);
  swap_tab();
  load_chunk(raX, rbX, last < 1 ? last : 1);
  load_tab(last < 2 ? last : 2);
  swap_tab();
  load_chunk(raY, rbY, last < 2 ? last : 2);
  load_tab(last < 3 ? last : 3);
  __syncthreads();
  auto iteration = [&](int kc, f64x2(&ra)[A_PER][2], double(&rb)[4]) {
    const int cur = kc & 1;
    swap_tab();  // entries of chunk kc + 3, fetched during the previous iteration
    store_chunk(ra, rb, cur ^ 1);
    load_chunk(ra, rb, kc + 3 < last ? kc + 3 : last);
    load_tab(kc + 4 < last ? kc + 4 : last);
    chunk_mfma<MB, NB, LDA, LDB>(opA + cur * STAGE, opB + cur * STAGE, acc);
    __syncthreads();
  };
  int kc = 0;
  for (; kc + 1 < nchunks; kc += 2) {
    iteration(kc, raX, rbX);
    iteration(kc + 1, raY, rbY);
  }
  if (kc < nchunks) iteration(kc, raX, rbX);

  // Epilogue.  One output phase per channel and an output of at most 2^30 bytes (see the fp32
  // epilogue): byte offsets per row and per column with out-of-range values for "not stored", and
  // range-checked buffer stores.
  // With a split reduction every slice writes its raw partial sums, in the output blob's own layout,
  // to its part of the workspace; reduce64_kernel adds them and the bias.
  double* const out = a.ksplit > 1 ? reinterpret_cast<double*>(a.part) + (size_t)split * a.out_elems
                                   : reinterpret_cast<double*>(a.out);
  const double* const bias = a.ksplit > 1 ? nullptr : reinterpret_cast<const double*>(a.bias);
  if (a.simple_epilogue) {
    uint32_t* rowoff = reinterpret_cast<uint32_t*>(smem);
    uint32_t* coloff = rowoff + BM;
    double* rbias = reinterpret_cast<double*>(coloff + BN);
    const double* bias8 = bias;
    if (t < BM) {
      const uint32_t gm = m_tile * BM + t;
      uint32_t off = 0x80000000u;
      double bb = 0.;
      if (gm < (uint32_t)a.Mrows) {
        const uint32_t chan = g * a.chan_per_grp + gm;
        off = 8u * chan * (uint32_t)(a.OHd * a.OWd);
        if (bias8) bb = bias8[chan];
      }
      rowoff[t] = off;
      rbias[t] = bb;
    } else if (t < BM + BN) {
      const int cl = t - BM;
      const uint32_t col = col_tile * BN + cl;
      uint32_t off = 0x40000000u;
      if (col < (uint32_t)a.ncols) {
        const uint32_t n = mdiv(col, a.mP);
        const uint32_t pix = col - n * a.P;
        const uint32_t pa = mdiv(pix, a.mPW);
        const uint32_t pb = pix - pa * a.PW;
        const int hh = (int)pa * a.OSh - a.opad_h, ww = (int)pb * a.OSw - a.opad_w;
        if ((uint32_t)hh < (uint32_t)a.OHd && (uint32_t)ww < (uint32_t)a.OWd)
          off = 8u * (n * (uint32_t)a.out_img_stride + (uint32_t)hh * (uint32_t)a.OWd + (uint32_t)ww);
      }
      coloff[cl] = off;
    }
    __syncthreads();
    const __amdgpu_buffer_rsrc_t out_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(out, 0, (int)(8u * (uint32_t)a.out_elems), 0x00020000);
    typedef int i32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const uint32_t co = coloff[(wn * NB + j) * 16 + (lane & 15)];
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int m = (wm * MB + i) * 16 + 4 * r + (lane >> 4);
          const double v = acc[i][j][r] + rbias[m];
          __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(i32x2, v), out_rsrc, rowoff[m] + co, 0, 0);
        }
    }
    return;
  }
  // General form: the same two LDS tables as the fp32 kernel (row -> channel / sub-pixel offset,
  // column -> image / pixel offset), the bias kept beside them as doubles.
  int4* rowtab = reinterpret_cast<int4*>(smem);
  int4* coltab = rowtab + BM;
  double* rowbias = reinterpret_cast<double*>(coltab + BN);
  if (t < BM) {
    const uint32_t gm = m_tile * BM + t;
    int off = 0, hh = -(1 << 28), ww = 0;
    double bb = 0.;
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
    rowtab[t] = make_int4(off, hh, ww, 0);
    rowbias[t] = bb;
  } else if (t < BM + BN) {
    const int cl = t - BM;
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
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const int4 ct = coltab[(wn * NB + j) * 16 + (lane & 15)];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int m = (wm * MB + i) * 16 + 4 * r + (lane >> 4);
        const int4 rt = rowtab[m];
        const int hh = rt.y + ct.y, ww = rt.z + ct.z;
        if ((uint32_t)hh < (uint32_t)a.OHd && (uint32_t)ww < (uint32_t)a.OWd)
          out[rt.x + ct.x] = acc[i][j][r] + rowbias[m];
      }
  }
}

// Backward filter: part[split][g][k][nn] = sum over the split's columns (n, oh, ow) of
// dy[n, g*Kg + k, oh, ow] * x[n, g*Cg + c, oh*sh - ph + i*dh, ow*sw - pw + j*dw], nn = (c, i, j).
// Lanes run along the reduction index (16 columns per chunk), 16 row slots per operand.
template <int MB, int NB, int WM, int WN>
__global__ __launch_bounds__(kThreads) void wgrad64_kernel(const WgradArgs a) {
  using C = Cfg64<MB, NB, WM, WN>;
  constexpr int BM = C::BM, STAGE = C::STAGE, LDA = C::LDA, LDB = C::LDB, AR = BM / 16;  // AR dy rows per thread
  __shared__ __align__(16) double smem[2 * STAGE];
  const int t = threadIdx.x, lane = t & 63;
  const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wv / WN, wn = wv % WN;
  const int kc = t & 15, rslot = t >> 4;

  uint32_t lin = xcd_contiguous_block_id();
  const uint32_t m_tile = lin % (uint32_t)a.m_tiles;
  lin /= (uint32_t)a.m_tiles;
  const uint32_t n_tile = lin % (uint32_t)a.n_tiles;
  lin /= (uint32_t)a.n_tiles;
  const uint32_t split = lin % (uint32_t)a.S;
  const uint32_t g = lin / (uint32_t)a.S;

  // rows this thread loads (rows past the matrix edge are clamped: they feed accumulators that
  // are never stored)
  uint32_t aoff[AR], boff[4], bij[4];
#pragma unroll
  for (int e = 0; e < AR; ++e) {
    uint32_t m = m_tile * BM + rslot + 16 * e;
    if (m > (uint32_t)a.Kg - 1) m = (uint32_t)a.Kg - 1;
    aoff[e] = 8u * m * (uint32_t)a.P;
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    uint32_t nn = n_tile * BN + rslot + 16 * e;
    if (nn > (uint32_t)a.Kred - 1) nn = (uint32_t)a.Kred - 1;
    const uint32_t c = mdiv(nn, a.mKHW);
    const uint32_t rem = nn - c * a.khw;
    const uint32_t i = mdiv(rem, a.mKW);
    const uint32_t j = rem - i * a.kw;
    boff[e] = 8u * ((g * a.Cg + c) * (uint32_t)a.HW + i * a.dh * a.W + j * a.dw);
    bij[e] = ((i * a.dh) << 16) | (j * a.dw);
  }
  const uint32_t c_begin = split * (uint32_t)a.cols_per_split;
  uint32_t c_end = c_begin + (uint32_t)a.cols_per_split;
  if (c_end > (uint32_t)a.ncols) c_end = (uint32_t)a.ncols;
  const int nchunks = c_begin < c_end ? (int)((c_end - c_begin + BK - 1) / BK) : 0;

  const __amdgpu_buffer_rsrc_t dy_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.dy), 0, (int)a.dy_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t x_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.x), 0, (int)a.x_bytes, 0x00020000);

  f64x4 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[i][j] = f64x4{0., 0., 0., 0.};

  // Two register sets: while chunk ch is multiplied out of one LDS buffer, the set holding chunk
  // ch+1 (loaded two iterations ago) goes to the other buffer and is reloaded with chunk ch+3; the
  // other set holds chunk ch+2.  Chunks past the end load nothing that is used (their columns fail
  // the range test and read as zero into a buffer nobody multiplies).
  double raX[AR], rbX[4], raY[AR], rbY[4];
  auto load_chunk = [&](double(&ra)[AR], double(&rb)[4], int chunk) {
    const uint32_t col = c_begin + chunk * BK + kc;
    const bool colok = col < c_end;
    const uint32_t n = mdiv(col, a.mP);
    const uint32_t pix = col - n * a.P;
    const uint32_t oh = mdiv(pix, a.mPW);
    const uint32_t ow = pix - oh * a.PW;
    const int ih0 = (int)oh * a.sh - a.ph;
    const int iw0 = (int)ow * a.sw - a.pw;
    const uint32_t dybase = 8u * ((n * a.Ktot + g * a.Kg) * (uint32_t)a.P + pix);
    const uint32_t xbase = 8u * (uint32_t)((int)(n * (uint32_t)(a.C * a.HW)) + ih0 * a.W + iw0);
#pragma unroll
    for (int e = 0; e < AR; ++e) ra[e] = buffer_load_f64(dy_rsrc, colok ? dybase + aoff[e] : a.dy_bytes);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int ih = ih0 + (int)(bij[e] >> 16), iw = iw0 + (int)(bij[e] & 0xffffu);
      const bool ok = colok & ((uint32_t)ih < (uint32_t)a.H) & ((uint32_t)iw < (uint32_t)a.W);
      rb[e] = buffer_load_f64(x_rsrc, ok ? xbase + boff[e] : a.x_bytes);
    }
  };
  auto store_chunk = [&](double(&ra)[AR], double(&rb)[4], int buf) {
#pragma unroll
    for (int e = 0; e < AR; ++e) smem[buf * STAGE + kc * LDA + rslot + 16 * e] = ra[e];
#pragma unroll
    for (int e = 0; e < 4; ++e) smem[buf * STAGE + BK * LDA + kc * LDB + rslot + 16 * e] = rb[e];
  };

  const double* opA = smem + (lane >> 4) * LDA + wm * MB * 16 + (lane & 15);
  const double* opB = smem + BK * LDA + (lane >> 4) * LDB + wn * NB * 16 + (lane & 15);
  if (nchunks > 0) {
    load_chunk(raX, rbX, 0);
    store_chunk(raX, rbX, 0);
    load_chunk(raX, rbX, 1);
    load_chunk(raY, rbY, 2);
  }
  __syncthreads();
  auto iteration = [&](int ch, double(&ra)[AR], double(&rb)[4]) {
    const int cur = ch & 1;
    store_chunk(ra, rb, cur ^ 1);  // chunk ch+1, in registers since iteration ch-2
    load_chunk(ra, rb, ch + 3);
    chunk_mfma<MB, NB, LDA, LDB>(opA + cur * STAGE, opB + cur * STAGE, acc);
    __syncthreads();
  };
  int ch = 0;
  for (; ch + 1 < nchunks; ch += 2) {
    iteration(ch, raX, rbX);
    iteration(ch + 1, raY, rbY);
  }
  if (ch < nchunks) iteration(ch, raX, rbX);

  double* dst = reinterpret_cast<double*>(a.part) + ((size_t)split * a.G + g) * ((size_t)a.Kg * a.Kred);
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const uint32_t nn = n_tile * BN + (wn * NB + j) * 16 + (lane & 15);
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const uint32_t k = m_tile * BM + (wm * MB + i) * 16 + 4 * r + (lane >> 4);
        if (k < (uint32_t)a.Kg && nn < (uint32_t)a.Kred) dst[(size_t)k * a.Kred + nn] = acc[i][j][r];
      }
  }
}

// dst = beta*dst + sum_s part[s] (+ bias), in a fixed order.  A workgroup owns 64 consecutive elements;
// its four waves each add a contiguous quarter of the slices (eight loads in flight per lane: a long
// run of slices is latency-bound otherwise) and the quarter sums are combined in wave order.
__global__ __launch_bounds__(256) void reduce64_kernel(const ReduceArgs a) {
  __shared__ double quarter[4][64];
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int i = (int)blockIdx.x * 64 + lane;
  const int per = (a.S + 3) / 4;
  const int s0 = q * per;
  int s1 = s0 + per;
  if (s1 > a.S) s1 = a.S;
  double acc[4] = {0., 0., 0., 0.};
  if (i < a.count) {
    const double* src = reinterpret_cast<const double*>(a.part) + i;
    int k = s0;
    for (; k + 7 < s1; k += 8) {
      double x[8];
#pragma unroll
      for (int c = 0; c < 8; ++c) x[c] = src[(size_t)(k + c) * a.count];
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[c & 3] += x[c];
    }
    for (; k < s1; ++k) acc[0] += src[(size_t)k * a.count];
  }
  quarter[q][lane] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
  __syncthreads();
  if (q != 0 || i >= a.count) return;
  double* dst = reinterpret_cast<double*>(a.dst);
  double v = ((quarter[0][lane] + quarter[1][lane]) + quarter[2][lane]) + quarter[3][lane];
  if (a.bias) {  // forward: channel of element i of an N x channels x chan_elems blob
    const uint32_t ch = mdiv((uint32_t)i, a.mChanElems);
    v += reinterpret_cast<const double*>(a.bias)[ch - mdiv(ch, a.mChannels) * (uint32_t)a.channels];
  }
  if (a.beta != 0.f) v += (double)a.beta * dst[i];
  dst[i] = v;
}

// part[s][k] = sum of dy[n][k][:] over the images of split s: one wave per image at a time.
__global__ __launch_bounds__(256) void bias_grad64_kernel(const BiasGradArgs a) {
  __shared__ double wsum[4];
  const int k = blockIdx.x, s = blockIdx.y;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int n0 = s * a.n_per_split;
  int n1 = n0 + a.n_per_split;
  if (n1 > a.N) n1 = a.N;
  const double* dy = reinterpret_cast<const double*>(a.dy);
  double acc0 = 0., acc1 = 0.;
  for (int n = n0 + wv; n < n1; n += 4) {
    const double* src = dy + ((size_t)n * a.K + k) * a.P;
    int p = lane;
    for (; p + 64 < a.P; p += 128) {
      acc0 += src[p];
      acc1 += src[p + 64];
    }
    for (; p < a.P; p += 64) acc0 += src[p];
  }
  double v = acc0 + acc1;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  if (lane == 0) wsum[wv] = v;
  __syncthreads();
  if (threadIdx.x == 0)
    reinterpret_cast<double*>(a.part)[(size_t)s * a.K + k] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
}

}  // namespace

// Row counts of the fp64 workgroup tiles (columns 64, k 16 for all of them).
// Ties go to the 64-row tile for the correlation (measured faster than 96 rows there: four
// workgroups per compute unit instead of three) and to the 96-row tile for the filter gradient.
int32_t f64_pick_rows(int64_t rows, bool filter_gradient) {
  static const int32_t corr_order[] = {64, 96, 48, 32, 16}, wgrad_order[] = {96, 64, 48, 32, 16};
  int32_t best = 64;
  int64_t best_pad = -1;
  for (int32_t bm : (filter_gradient ? wgrad_order : corr_order)) {
    const int64_t pad = (rows + bm - 1) / bm * bm;
    if (best_pad < 0 || pad < best_pad) {
      best = bm;
      best_pad = pad;
    }
  }
  return best;
}

int launch_corr64(int32_t bm, const CorrArgs& a, void* stream) {
  const dim3 grid((uint32_t)a.G * a.m_tiles * a.col_tiles * (a.ksplit > 1 ? a.ksplit : 1)), block(kThreads);
  hipStream_t s = (hipStream_t)stream;
  switch (bm) {
    case 96: hipLaunchKernelGGL((corr64_kernel<3, 2, 2, 2>), grid, block, 0, s, a); break;
    case 64: hipLaunchKernelGGL((corr64_kernel<2, 2, 2, 2>), grid, block, 0, s, a); break;
    case 48: hipLaunchKernelGGL((corr64_kernel<3, 1, 1, 4>), grid, block, 0, s, a); break;
    case 32: hipLaunchKernelGGL((corr64_kernel<2, 1, 1, 4>), grid, block, 0, s, a); break;
    case 16: hipLaunchKernelGGL((corr64_kernel<1, 1, 1, 4>), grid, block, 0, s, a); break;
    default: return (int)hipErrorInvalidValue;
  }
  return (int)hipGetLastError();
}

int launch_wgrad64(int32_t bm, const WgradArgs& a, void* stream) {
  const dim3 grid((uint32_t)a.G * a.S * a.m_tiles * a.n_tiles), block(kThreads);
  hipStream_t s = (hipStream_t)stream;
  switch (bm) {
    case 96: hipLaunchKernelGGL((wgrad64_kernel<3, 2, 2, 2>), grid, block, 0, s, a); break;
    case 64: hipLaunchKernelGGL((wgrad64_kernel<2, 2, 2, 2>), grid, block, 0, s, a); break;
    case 48: hipLaunchKernelGGL((wgrad64_kernel<3, 1, 1, 4>), grid, block, 0, s, a); break;
    case 32: hipLaunchKernelGGL((wgrad64_kernel<2, 1, 1, 4>), grid, block, 0, s, a); break;
    case 16: hipLaunchKernelGGL((wgrad64_kernel<1, 1, 1, 4>), grid, block, 0, s, a); break;
    default: return (int)hipErrorInvalidValue;
  }
  return (int)hipGetLastError();
}

int launch_reduce64(const ReduceArgs& a, void* stream) {
  hipLaunchKernelGGL(reduce64_kernel, dim3((a.count + 63) / 64), dim3(256), 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

int launch_bias_grad64(const BiasGradArgs& a, void* stream) {
  hipLaunchKernelGGL(bias_grad64_kernel, dim3(a.K, a.S), dim3(256), 0, (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

}  // namespace mi355conv
