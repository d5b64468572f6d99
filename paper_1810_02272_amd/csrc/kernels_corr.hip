// Implicit-GEMM correlation kernel for gfx950, used by the forward pass and (through the
// sub-pixel rewriting of the transposed map) by the backward-data pass of the Caffe-semantics
// convolution layer (paper Table 1, "vision layers"; lowering + GEMM + bias are the steps the
// low-level math library of the paper's "General Architecture" section performs).
//
//   D[m][col] = sum_kk A[m][kk] * B[kk][col]
//   B[kk][col] = in[n, g*Cg + c, a*sh - ph + i*dh, b*sw - pw + j*dw]  (0 outside the image)
//   kk = (c, i, j), col = (n, a, b)
//
// B is never materialised: each workgroup gathers BK x BN elements of it straight from the NCHW
// blob through registers into a two-stage LDS ring, two chunks ahead of the fp32 MFMA pipe.  A is
// the weight matrix, packed beforehand into zero-padded [row][k] form so that its tiles are plain
// 16-byte copies.  The epilogue adds the bias and scatters each accumulator through two
// small LDS tables (row -> channel/sub-pixel offset, column -> image/pixel offset), which is
// what lets one kernel serve both passes.
#include <hip/hip_runtime.h>

#include "corr_epilogue.h"
#include "device_utils.h"
#include "internal.h"

namespace mi355conv {

namespace {

constexpr int kThreads = 256;

template <int MT, int MB, int NB, int WM, int WN, int BK>
struct CorrCfg {
  static constexpr int BM = WM * MB * MT;
  static constexpr int BN = WN * NB * MT;
  // Both LDS tiles are [row][k], 16-byte aligned rows.  32-row MFMA: rows of BK + 4 floats -- the
  // 16-byte operand reads (lanes 0..31 on 32 consecutive rows) and the 16-byte staging writes are
  // conflict free.  16-row MFMA: a wave's operand read covers 16 rows x 4 k quads, which on rows of
  // BK + 4 floats takes twice the cycles (measured with the bank-conflict counter on a probe
  // kernel); rows of BK + 8 floats with the position of a row's k quad XORed with bit 2 of the row
  // number make that read and both staging writes conflict free.
  static constexpr int LDK = MT == 16 ? BK + 8 : BK + 4;
  static constexpr bool SWZ = MT == 16;
  static constexpr int RPW = 4;        // gathered k rows per wave and chunk: one 16-byte LDS write
  static constexpr int CPL = BN / 64;  // gathered columns per lane
  static constexpr int A_WI = BM / 16;  // wave-wide 16-byte loads per chunk of A (16 rows x 16 k each)
  static constexpr int A_PER = (A_WI + 3) / 4;
  static constexpr int STAGE = (BM + BN) * LDK;  // floats per pipeline stage
  static constexpr int SMEM = 2 * STAGE;
  static constexpr int KSS = 4 * (64 / MT);  // k values covered by one 16-byte operand read of a wave
  static constexpr int NSS = BK / KSS;
  static constexpr int NKS = BK / Mfma<MT>::KS;  // MFMA k steps per chunk
  static_assert(WM * WN == 4, "four waves per workgroup");
  static_assert(BK == 16, "each wave gathers one quad of k rows per chunk");
  static_assert(BN % 64 == 0 && BM % 16 == 0, "tile shape");
  static_assert(4 * (BM + BN) <= SMEM, "epilogue tables reuse the pipeline buffers");
};

// MODE: how a gathered element is bounds-checked (see the gather below): 0 no padding, 1 row and
// column compares, 2 per-column tap bitmask.
template <int MT, int MB, int NB, int WM, int WN, int BK, int MODE>
__global__ __launch_bounds__(kThreads) void corr_kernel(const CorrArgs a) {
  using C = CorrCfg<MT, MB, NB, WM, WN, BK>;
  using M = Mfma<MT>;
  constexpr int BM = C::BM, BN = C::BN, LDK = C::LDK, RPW = C::RPW, CPL = C::CPL;

  __shared__ __align__(16) float smem[C::SMEM];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wv / WN, wn = wv % WN;

  // tile coordinates: m tile fastest, then column tile, then group
  uint32_t lin = xcd_contiguous_block_id();
  const uint32_t m_tile = lin % (uint32_t)a.m_tiles;
  lin /= (uint32_t)a.m_tiles;
  const uint32_t col_tile = lin % (uint32_t)a.col_tiles;
  lin /= (uint32_t)a.col_tiles;
  const uint32_t g = lin % (uint32_t)a.G;
  const uint32_t split = lin / (uint32_t)a.G;  // which part of the reduction (split-K; usually the only one)

  // Per-lane column state of the gather (fixed for the whole reduction).  An element that must
  // read as zero -- tap in the padding, column past the edge, k row past the reduction length --
  // is given an offset at or beyond the buffer size, and the hardware range check of the buffer
  // load returns 0 for it.  Three ways to get there:
  //  MODE 0 (no padding: every tap of a real column is inside the image; buffer < 2^31 bytes):
  //    nothing per element -- an invalid column has base 2^31, an invalid k row has offset
  //    2^31 - 4 in the k table.
  //  MODE 1 (general): row and column compares per element, select the buffer size.
  //  MODE 2 (at most 32 taps; buffer <= 2^29 bytes): whether tap t is outside the image depends
  //    only on the column, so each lane keeps one bitmask per column and adds bit t of it, shifted
  //    to 2^31, to the offset (an invalid k row has offset 2^30 in the k table).
  uint32_t cbase[CPL];
  int cih0[CPL], ciw0[CPL];
  uint32_t cinv[CPL];
  uint32_t row_bits = 0;  // bit i*TW for every tap row i (MODE 2)
  if (MODE == 2)
    for (int i = 0; i < a.THW / a.TW; ++i) row_bits |= 1u << (i * a.TW);
#pragma unroll
  for (int q = 0; q < CPL; ++q) {
    const uint32_t col = col_tile * BN + q * 64 + lane;
    if (col < (uint32_t)a.ncols) {
      const uint32_t n = mdiv(col, a.mP);
      const uint32_t pix = col - n * a.P;
      const uint32_t pa = mdiv(pix, a.mPW);
      const uint32_t pb = pix - pa * a.PW;
      const int ih0 = (int)pa * a.sh - a.ph;
      const int iw0 = (int)pb * a.sw - a.pw;
      cih0[q] = ih0;
      ciw0[q] = iw0;
      cbase[q] = 4u * (uint32_t)((int)(n * a.in_img_stride + g * a.in_grp_stride) + ih0 * a.IW + iw0);
    } else {
      cih0[q] = -(1 << 29);  // every bounds test fails, also with the 2^28 of an invalid k row
      ciw0[q] = 0;
      cbase[q] = MODE == 0 ? 0x80000000u : 0u;
    }
    cinv[q] = 0;
    if (MODE == 2) {
      const int TH = a.THW / a.TW;
      if (a.dh == 1 && a.dw == 1) {
        // The taps inside the image are i in [lo, hi) x j in [lo, hi): the mask over the tap index
        // i*TW + j is (bits lo..hi-1 of the column range) times (bit i*TW for every valid i) -- the
        // shifted copies of the column mask do not overlap, so one multiply builds the outer product.
        auto bit = [](int n) { return n >= 32 ? 0u : 1u << n; };  // 2^n modulo 2^32
        int lo = -cih0[q], hi = a.IH - cih0[q];
        lo = lo < 0 ? 0 : (lo > TH ? TH : lo);
        hi = hi < lo ? lo : (hi > TH ? TH : hi);
        const uint32_t rows = row_bits & (bit(hi * a.TW) - bit(lo * a.TW));
        lo = -ciw0[q], hi = a.IW - ciw0[q];
        lo = lo < 0 ? 0 : (lo > a.TW ? a.TW : lo);
        hi = hi < lo ? lo : (hi > a.TW ? a.TW : hi);
        cinv[q] = ~((bit(hi) - bit(lo)) * rows);
      } else {
        for (int i = 0, tap = 0; i < TH; ++i)
          for (int j = 0; j < a.TW; ++j, ++tap) {
            const bool ok = ((uint32_t)(cih0[q] + i * a.dh) < (uint32_t)a.IH) &
                            ((uint32_t)(ciw0[q] + j * a.dw) < (uint32_t)a.IW);
            cinv[q] |= ok ? 0u : (1u << tap);
          }
      }
    }
  }

  // A tile: [row][k], 16 bytes (four k) per lane; a wave-wide load covers 16 rows x 16 k with
  // 8 consecutive lanes on 8 consecutive rows (conflict-free LDS write, 64-byte runs in memory).
  const int kc_first = (int)split * a.chunks_per_split;
  const float* Ag = a.A + ((size_t)g * a.MP + (size_t)m_tile * BM) * a.KP + (size_t)kc_first * BK;
  const int arow = (lane & 7) + 8 * (lane >> 5), ac4 = (lane >> 3) & 3;
  const int aswz = C::SWZ ? (arow >> 2) & 1 : 0, bswz = C::SWZ ? (lane >> 2) & 1 : 0;  // k-quad swizzle of this lane's rows
  uint32_t aoff[C::A_PER];
#pragma unroll
  for (int p = 0; p < C::A_PER; ++p) aoff[p] = 4u * (uint32_t)(((wv + 4 * p) * 16 + arow) * a.KP + ac4 * 4);

  const __amdgpu_buffer_rsrc_t in_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.in), 0, (int)a.in_bytes, 0x00020000);

  typename M::Acc acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < M::NR; ++r) acc[i][j][r] = 0.f;

  // Two register sets for the staged operands: chunks k+1 and k+2 are both in flight while chunk k
  // is multiplied, so a load has two full iterations to arrive before its LDS write needs it.
  // Element e of rb[q]: k row 4*wv + e of column q*64 + lane.
  f32x4 raX[C::A_PER], raY[C::A_PER];
  f32x4 rbX[CPL], rbY[CPL];

  auto load_a = [&](f32x4(&ra)[C::A_PER], int kc, int p) {
    if (C::A_WI % 4 == 0 || wv + 4 * p < C::A_WI)
      ra[p] = *reinterpret_cast<const f32x4*>(reinterpret_cast<const char*>(Ag) + (aoff[p] + (uint32_t)kc * (BK * 4)));
  };
  auto store_a = [&](f32x4(&ra)[C::A_PER], int buf, int p) {
    if (C::A_WI % 4 == 0 || wv + 4 * p < C::A_WI)
      *reinterpret_cast<f32x4*>(smem + buf * C::STAGE + ((wv + 4 * p) * 16 + arow) * LDK + (ac4 ^ aswz) * 4) = ra[p];
  };
  // Rows of this wave in a chunk: each tap's byte offset and (row, column) displacement come from
  // the k table with scalar loads (the index is uniform over the wave).  The entries are fetched a
  // whole iteration before their use, in the middle of a chunk's MFMAs, so that the scalar-memory
  // latency never sits in front of an MFMA or the barrier.
  KTabEntry te[RPW], te_next[RPW];
  auto load_tab = [&](int kc) {
#pragma unroll
    for (int e = 0; e < RPW; ++e) te_next[e] = a.ktab[(kc_first + kc) * BK + wv * RPW + e];
  };
  auto swap_tab = [&]() {
#pragma unroll
    for (int e = 0; e < RPW; ++e) te[e] = te_next[e];
  };
  auto load_b = [&](f32x4(&rb)[CPL], int q, int e) {
    uint32_t off = cbase[q] + te[e].koff;
    if (MODE == 1) {
      const int ih = cih0[q] + te[e].idh, iw = ciw0[q] + te[e].jdw;
      const bool ok = ((uint32_t)ih < (uint32_t)a.IH) & ((uint32_t)iw < (uint32_t)a.IW);
      off = ok ? off : a.in_bytes;  // the buffer size: first byte past the end, no 32-bit wrap
    } else if (MODE == 2) {
      off += __builtin_amdgcn_ubfe(cinv[q], (uint32_t)te[e].tap, 1u) << 31;
    }
    rb[q][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(in_rsrc, off, 0, 0));
  };
  auto store_b = [&](f32x4(&rb)[CPL], int buf, int q) {
    *reinterpret_cast<f32x4*>(smem + buf * C::STAGE + BM * LDK + (q * 64 + lane) * LDK + (wv ^ bswz) * 4) = rb[q];
  };
  // Software pipeline, four chunks deep: while the MFMA pipe works on chunk k out of one LDS buffer,
  // the register set holding chunk k+1 (loaded two iterations ago) is written to the other buffer
  // and immediately reloaded with chunk k+3; the other register set holds chunk k+2 meanwhile.
  // The stores and loads are spread over the k steps of the chunk so that their address
  // arithmetic issues in the shadow of the MFMAs of the same wave.  Chunk indices past the end
  // are clamped: the last iterations re-load and re-store the final chunk into a buffer nobody
  // reads.
  //
  // MFMA operands come from LDS as 16-byte reads: lane l takes row l%MT and the four k values
  // KSS*s + 4*(l/MT) .. +3, which feed four consecutive MFMAs; the k order inside a group of KSS
  // is thereby permuted, identically for both operands, which a sum does not notice.
  int nchunks = a.KP / BK - kc_first;  // chunks of this split (chunk indices below are relative to it)
  if (nchunks > a.chunks_per_split) nchunks = a.chunks_per_split;
  const int last = nchunks - 1;
  constexpr int NKS = C::NKS, NSS = C::NSS;
  const int oswz = C::SWZ ? ((lane % MT) >> 2) & 1 : 0;
  const float* opA = smem + (wm * MB * MT + lane % MT) * LDK + ((lane / MT) ^ oswz) * 4;
  const float* opB = smem + BM * LDK + (wn * NB * MT + lane % MT) * LDK + ((lane / MT) ^ oswz) * 4;

  // Prologue: the table entries of the first three chunks are requested together (one scalar-memory
  // round trip instead of three in a row), then each chunk's operand loads use its own entries.
  KTabEntry first[3][RPW];
#pragma unroll
  for (int c = 0; c < 3; ++c)
#pragma unroll
    for (int e = 0; e < RPW; ++e) first[c][e] = a.ktab[(kc_first + (last < c ? last : c)) * BK + wv * RPW + e];
  auto load_first = [&](f32x4(&ra)[C::A_PER], f32x4(&rb)[CPL], int c) {
#pragma unroll
    for (int e = 0; e < RPW; ++e) te[e] = first[c][e];
#pragma unroll
    for (int p = 0; p < C::A_PER; ++p) load_a(ra, last < c ? last : c, p);
#pragma unroll
    for (int q = 0; q < CPL; ++q)
#pragma unroll
      for (int e = 0; e < RPW; ++e) load_b(rb, q, e);
  };
  load_first(raX, rbX, 0);
#pragma unroll
  for (int p = 0; p < C::A_PER; ++p) store_a(raX, 0, p);
#pragma unroll
  for (int q = 0; q < CPL; ++q) store_b(rbX, 0, q);
  load_first(raX, rbX, 1);
  load_first(raY, rbY, 2);
  load_tab(last < 3 ? last : 3);
  __syncthreads();

  auto iteration = [&](int kc, f32x4(&ra)[C::A_PER], f32x4(&rb)[CPL]) {
    const int cur = kc & 1, nxt = cur ^ 1;
    const int kld = kc + 3 < last ? kc + 3 : last;
    swap_tab();  // entries for this iteration's loads (chunk kc + 3) arrived during the previous one
    const float* sA = opA + cur * C::STAGE;
    const float* sB = opB + cur * C::STAGE;
    f32x4 av[2][MB], bv[2][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i) av[0][i] = *reinterpret_cast<const f32x4*>(sA + i * MT * LDK);
#pragma unroll
    for (int j = 0; j < NB; ++j) bv[0][j] = *reinterpret_cast<const f32x4*>(sB + j * MT * LDK);
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      const int ss = ks / 4, u = ks % 4;
      if (u == 0 && ss + 1 < NSS) {  // operands of the next group of four steps
#pragma unroll
        for (int i = 0; i < MB; ++i)
          av[(ss + 1) & 1][i] = *reinterpret_cast<const f32x4*>(sA + i * MT * LDK + (ss + 1) * C::KSS);
#pragma unroll
        for (int j = 0; j < NB; ++j)
          bv[(ss + 1) & 1][j] = *reinterpret_cast<const f32x4*>(sB + j * MT * LDK + (ss + 1) * C::KSS);
      }
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) M::run(av[ss & 1][i][u], bv[ss & 1][j][u], acc[i][j]);
      // Table entries for the next iteration's loads.  Scalar loads share the LDS counter and return
      // out of order, so any LDS wait behind them becomes a full wait: they are issued in the middle
      // of the chunk, one step after the last operand read of this iteration was consumed, and have half a
      // chunk of MFMAs to arrive before the barrier's wait.
      if (ks == (NSS > 1 ? NKS / 2 + 1 : 1)) load_tab(kc + 4 < last ? kc + 4 : last);
      // this step's share of the staging work
#pragma unroll
      for (int q = 0; q < CPL; ++q)
#pragma unroll
        for (int e = 0; e < RPW; ++e)
          if ((q * RPW + e) * NKS / (CPL * RPW) == ks) {
            if (e == 0) store_b(rb, nxt, q);
            load_b(rb, q, e);
          }
#pragma unroll
      for (int p = 0; p < C::A_PER; ++p)
        if ((p * NKS + NKS / 2) / C::A_PER % NKS == ks) {
          store_a(ra, nxt, p);
          load_a(ra, kld, p);
        }
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
  };

  int kc = 0;
  for (; kc + 1 < nchunks; kc += 2) {
    iteration(kc, raX, rbX);
    iteration(kc + 1, raY, rbY);
  }
  if (kc < nchunks) iteration(kc, raX, rbX);

  corr_epilogue<MT, MB, NB, BM, BN>(a, smem, acc, m_tile, col_tile, g, wm, wn, split);
}

// One k-table entry: where tap kk = (c, i, j) of the gather sits relative to a column's base.
__device__ __forceinline__ void fill_ktab(const PackArgs& a, int kk) {
  const int c = kk / a.tTHW, rem = kk % a.tTHW;
  const int i = rem / a.tTW, j = rem % a.tTW;
  KTabEntry e;
  // k rows past the reduction length fail the row test and carry the offset that the kernel's
  // bounds mode needs to land beyond the buffer
  e.koff = kk < a.Kred ? 4u * (uint32_t)(c * a.tIHW + i * a.tdh * a.tIW + j * a.tdw) : a.koff_invalid;
  e.idh = kk < a.Kred ? i * a.tdh : (1 << 28);
  e.jdw = j * a.tdw;
  e.tap = rem & 31;
  a.ktab[kk] = e;
}

// Divisors of the pack kernels' index arithmetic as magic numbers (built per launch on the host).
struct PackMagic {
  Magic KP, MP, perm, QQ, Qw, nv, nvw, dh, dw;
};

// Packed position kp -> reduction index (channel, tap) in the blob's own order.  The patch kernel
// runs the reduction as (8-channel chunk, tap, channel in chunk); the gather kernel keeps (c, tap).
__device__ __forceinline__ int source_k(const PackArgs& a, const PackMagic& mg, int kp) {
  if (a.kperm_T == 0) return kp;
  const int T = a.kperm_T;
  const int cc = (int)mdiv((uint32_t)kp, mg.perm), rem = kp - cc * 8 * T;
  return (cc * 8 + (rem & 7)) * T + (rem >> 3);
}

// Forward: A[g][m][k] = w[g*Kg + m][k], zero padded to [MP][KP] (the weight blob's own order).
// T is the base type of the blob (the pointer members of PackArgs address floats or doubles).
template <typename T>
__global__ __launch_bounds__(256) void pack_fwd_kernel(const PackArgs a, const PackMagic mg) {
  const uint32_t total = (uint32_t)a.G * (uint32_t)a.MP * (uint32_t)a.KP;
  const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
  if (idx >= total) return;
  const uint32_t row = mdiv(idx, mg.KP);
  const int kp = (int)(idx - row * (uint32_t)a.KP);
  const int g = (int)mdiv(row, mg.MP);
  const int m = (int)(row - (uint32_t)g * (uint32_t)a.MP);
  const int kk = source_k(a, mg, kp);
  const T* w = reinterpret_cast<const T*>(a.w);
  reinterpret_cast<T*>(a.A)[idx] = (m < a.Mrows && kp < a.Kred) ? w[((size_t)g * a.Kg + m) * a.Kred + kk] : T(0);
  if (m == 0 && g == 0) fill_ktab(a, kp);
}

// Backward data: rows are (input channel, row phase, column phase), k is (output channel,
// flipped reduced tap).  Phase (rh, rw) of input position h + pad = stride*a + rh is reached by
// tap i exactly when i*dilation = stride*q + rh for an integer q >= 0; the gather then reads
// dy at a - q.  Only phases that some tap reaches have rows (the others are zero-filled by the
// host code), and when the stride divides the dilation -- stride 1 included -- the taps sit eh =
// dilation/stride rows of dy apart, so slot qh stands for q = qh*eh.  Entries with no such tap
// are zero.
template <typename T>
__global__ __launch_bounds__(256) void pack_bwd_kernel(const PackArgs a, const PackMagic mg) {
  const uint32_t total = (uint32_t)a.G * (uint32_t)a.MP * (uint32_t)a.KP;
  const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
  if (idx >= total) return;
  const uint32_t row = mdiv(idx, mg.KP);
  const int kp = (int)(idx - row * (uint32_t)a.KP);
  const int g = (int)mdiv(row, mg.MP);
  const int m = (int)(row - (uint32_t)g * (uint32_t)a.MP);
  const int kk = source_k(a, mg, kp);
  const T* w = reinterpret_cast<const T*>(a.w);
  T v = T(0);
  if (m < a.Mrows && kp < a.Kred) {
    const int QQ = a.Qh * a.Qw;
    const int k = (int)mdiv((uint32_t)kk, mg.QQ), qr = kk - k * QQ;
    const int qrh = (int)mdiv((uint32_t)qr, mg.Qw);
    const int qh = a.Qh - 1 - qrh, qw = a.Qw - 1 - (qr - qrh * a.Qw);
    const int nv = a.nvh * a.nvw;
    const int c = (int)mdiv((uint32_t)m, mg.nv), mr = m - c * nv;
    int rh = (int)mdiv((uint32_t)mr, mg.nvw), rw = mr - rh * a.nvw;
    if (a.tab_h) rh = a.phase_h[rh];
    if (a.tab_w) rw = a.phase_w[rw];
    const int th = a.sh * a.eh * qh + rh, tw = a.sw * a.ew * qw + rw;
    const int i = (int)mdiv((uint32_t)th, mg.dh), j = (int)mdiv((uint32_t)tw, mg.dw);
    if (i * a.dh == th && j * a.dw == tw && i < a.kh && j < a.kw)
      v = w[((((size_t)g * a.Kg + k) * a.Cg + c) * a.kh + i) * a.kw + j];
  }
  reinterpret_cast<T*>(a.A)[idx] = v;
  if (m == 0 && g == 0) fill_ktab(a, kp);
}

template <int MT, int MB, int NB, int WM, int WN, int BK>
int launch_corr_t(const CorrArgs& a, hipStream_t s) {
  const uint32_t blocks = (uint32_t)a.G * a.m_tiles * a.col_tiles * a.ksplit;
  if (a.bounds_mode == 0)
    hipLaunchKernelGGL((corr_kernel<MT, MB, NB, WM, WN, BK, 0>), dim3(blocks), dim3(kThreads), 0, s, a);
  else if (a.bounds_mode == 2)
    hipLaunchKernelGGL((corr_kernel<MT, MB, NB, WM, WN, BK, 2>), dim3(blocks), dim3(kThreads), 0, s, a);
  else
    hipLaunchKernelGGL((corr_kernel<MT, MB, NB, WM, WN, BK, 1>), dim3(blocks), dim3(kThreads), 0, s, a);
  return (int)hipGetLastError();
}

}  // namespace

void corr_tile_shape(int32_t tile, int32_t* bm, int32_t* bn, int32_t* bk) {
  static const int32_t shapes[CORR_TILE_COUNT][3] = {
      {128, 128, 16}, {128, 64, 16}, {96, 128, 16}, {64, 128, 16}, {64, 64, 16},
      {32, 256, 16},  {32, 128, 16}, {48, 256, 16}, {48, 128, 16}, {16, 256, 16}, {16, 64, 16}};
  *bm = shapes[tile][0];
  *bn = shapes[tile][1];
  *bk = shapes[tile][2];
}

const char* corr_tile_name(int32_t tile) {
  static const char* names[CORR_TILE_COUNT] = {
      "corr_m32_128x128x16", "corr_m32_128x64x16", "corr_m32_96x128x16",
      "corr_m32_64x128x16",  "corr_m32_64x64x16",  "corr_m32_32x256x16", "corr_m32_32x128x16",
      "corr_m16_48x256x16",  "corr_m16_48x128x16", "corr_m16_16x256x16", "corr_m16_16x64x16"};
  return names[tile];
}

int launch_corr(int32_t tile, const CorrArgs& a, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  switch (tile) {  //                      MT MB NB WM WN BK
    case CORR_128x128: return launch_corr_t<32, 2, 2, 2, 2, 16>(a, s);
    case CORR_128x64:  return launch_corr_t<32, 2, 1, 2, 2, 16>(a, s);
    case CORR_96x128:  return launch_corr_t<32, 3, 1, 1, 4, 16>(a, s);
    case CORR_64x128:  return launch_corr_t<32, 2, 1, 1, 4, 16>(a, s);
    case CORR_64x64:   return launch_corr_t<32, 1, 1, 2, 2, 16>(a, s);
    case CORR_32x256:  return launch_corr_t<32, 1, 2, 1, 4, 16>(a, s);
    case CORR_32x128:  return launch_corr_t<32, 1, 1, 1, 4, 16>(a, s);
    case CORR_48x256:  return launch_corr_t<16, 3, 4, 1, 4, 16>(a, s);
    case CORR_48x128:  return launch_corr_t<16, 3, 2, 1, 4, 16>(a, s);
    case CORR_16x256:  return launch_corr_t<16, 1, 4, 1, 4, 16>(a, s);
    case CORR_16x64:   return launch_corr_t<16, 1, 1, 1, 4, 16>(a, s);
    default: return (int)hipErrorInvalidValue;
  }
}

int launch_pack(const PackArgs& a, void* stream, bool f64) {
  hipStream_t s = (hipStream_t)stream;
  const size_t total = (size_t)a.G * a.KP * a.MP;
  const dim3 grid((uint32_t)((total + 255) / 256));
  auto positive = [](int32_t v) { return (uint32_t)(v > 0 ? v : 1); };
  PackMagic mg;
  mg.KP = make_magic(positive(a.KP));
  mg.MP = make_magic(positive(a.MP));
  mg.perm = make_magic(positive(8 * a.kperm_T));
  mg.QQ = make_magic(positive(a.Qh * a.Qw));
  mg.Qw = make_magic(positive(a.Qw));
  mg.nv = make_magic(positive(a.nvh * a.nvw));
  mg.nvw = make_magic(positive(a.nvw));
  mg.dh = make_magic(positive(a.dh));
  mg.dw = make_magic(positive(a.dw));
  if (a.mode == 0) {
    if (f64)
      hipLaunchKernelGGL(pack_fwd_kernel<double>, grid, dim3(256), 0, s, a, mg);
    else
      hipLaunchKernelGGL(pack_fwd_kernel<float>, grid, dim3(256), 0, s, a, mg);
  } else {
    if (f64)
      hipLaunchKernelGGL(pack_bwd_kernel<double>, grid, dim3(256), 0, s, a, mg);
    else
      hipLaunchKernelGGL(pack_bwd_kernel<float>, grid, dim3(256), 0, s, a, mg);
  }
  return (int)hipGetLastError();
}

}  // namespace mi355conv
