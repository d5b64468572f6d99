// Backward-filter kernel for gfx950 (Caffe-semantics convolution layer, paper Table 1):
//   dW_g[k][(c,i,j)] = sum over columns (n,oh,ow) of dy[n, g*Kg + k, oh, ow] *
//                      x[n, g*Cg + c, oh*sh - ph + i*dh, ow*sw - pw + j*dw]   (0 outside the image)
// an implicit GEMM whose reduction runs over the N*OH*OW output positions.  The output is tiny and
// the reduction huge, so the reduction is split over workgroups (split-K); every split writes its
// partial tile to the workspace and a second kernel adds the partials in a fixed order, which
// keeps the result deterministic (no float atomics) and applies beta.
//
// Both operands are read with lanes along the reduction index (contiguous in dy, contiguous for
// stride-1 x) and written to LDS as [row][k].  The MFMA operands come back as 16-byte reads:
// lane l takes row l%32 and the four k values 8t + 4(l/32) .. +3, which feed four consecutive
// 32x32x2 instructions -- the k order inside a group of eight is permuted, identically for both
// operands, which a sum does not notice.
//
// Two staging forms.  Through registers: a thread's loads return into registers and are stored to
// LDS one chunk later (three chunks in flight).  Straight to LDS (the 128x128 tile): the buffer loads
// write LDS themselves -- lane l of a wave fills word l of a 64-word segment, i.e. one row pair --
// with out-of-range lanes writing the zero the range check returns; no staging registers and no LDS
// store instructions, two chunks in flight, and a wait for the wave's own loads before each barrier.
#include <hip/hip_runtime.h>

#include "device_utils.h"
#include "internal.h"

namespace mi355conv {

namespace {

constexpr int kThreads = 256;

template <int MB, int NB, int WM, int WN, bool DMA = false>
struct WgCfg {
  static constexpr int MT = 32;
  static constexpr int BK = 32;
  static constexpr int BM = WM * MB * MT;
  static constexpr int BN = WN * NB * MT;
  // Register staging: rows of BK + 4 floats (16-byte aligned; 8 consecutive rows start on 8 distinct
  // bank quads).  Loads that write LDS themselves put the 64 lanes of a wave -- two rows of 32 k
  // values -- into 64 consecutive words, so rows come in pairs: a pair takes 2*BK + 4 floats, which
  // again spreads 16 consecutive rows over the 16 bank quads.
  static constexpr int LDK = BK + 4;
  static constexpr int PAIR = 2 * BK + 4;
  static constexpr int A_PER = BM / 8;  // rows per thread: 32 lanes along k, 8 row slots
  static constexpr int B_PER = BN / 8;
  static constexpr int A_FLOATS = DMA ? BM / 2 * PAIR : BM * LDK;
  static constexpr int STAGE = DMA ? (BM + BN) / 2 * PAIR : (BM + BN) * LDK;
  static constexpr int SMEM_BYTES = 2 * STAGE * 4;
  static_assert(WM * WN == 4, "four waves per workgroup");
  // float offset of row r inside an operand's tile
  static constexpr __device__ int row_off(int r) { return DMA ? (r >> 1) * PAIR + (r & 1) * BK : r * LDK; }
};

typedef __attribute__((address_space(3))) void* LdsPtr;

// MODE: how a gathered x element is bounds-checked, as in the correlation kernel: 0 no padding,
// 1 row and column compares, 2 per-column tap bitmask (dilation 1, at most 16 taps per dimension and
// 32 in all, blobs at most 2^29 bytes).
// DMA: the loads write LDS themselves (no register staging, no LDS store instructions); the pipeline
// is then two chunks deep -- chunk ch+1 lands in the other buffer while chunk ch is multiplied.
template <int MB, int NB, int WM, int WN, int MODE, bool DMA>
__global__ __launch_bounds__(kThreads) void wgrad_kernel(const WgradArgs a) {
  using C = WgCfg<MB, NB, WM, WN, DMA>;
  using M = Mfma<32>;
  constexpr int BM = C::BM, BN = C::BN, BK = C::BK, LDK = C::LDK, A_PER = C::A_PER, B_PER = C::B_PER;

  extern __shared__ __align__(16) float smem[];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wv / WN, wn = wv % WN;
  const int kc = t & 31, rslot = t >> 5;

  // tile coordinates: (m tile, n tile) fastest so that neighbours share the same columns
  uint32_t lin = xcd_contiguous_block_id();
  const uint32_t m_tile = lin % (uint32_t)a.m_tiles;
  lin /= (uint32_t)a.m_tiles;
  const uint32_t n_tile = lin % (uint32_t)a.n_tiles;
  lin /= (uint32_t)a.n_tiles;
  const uint32_t split = lin % (uint32_t)a.S;
  const uint32_t g = lin / (uint32_t)a.S;

  // Rows this thread loads, fixed for the whole kernel.  Rows past the matrix edge are clamped to
  // the last real row: they only feed accumulators that are never stored.
  uint32_t aoff[A_PER];
#pragma unroll
  for (int e = 0; e < A_PER; ++e) {
    uint32_t m = m_tile * BM + rslot + 8 * e;
    if (m > (uint32_t)a.Kg - 1) m = (uint32_t)a.Kg - 1;
    aoff[e] = 4u * m * (uint32_t)a.P;
  }
  uint32_t boff[B_PER], bij[B_PER];
#pragma unroll
  for (int e = 0; e < B_PER; ++e) {
    uint32_t nn = n_tile * BN + rslot + 8 * e;
    if (nn > (uint32_t)a.Kred - 1) nn = (uint32_t)a.Kred - 1;
    const uint32_t c = mdiv(nn, a.mKHW);
    const uint32_t rem = nn - c * a.khw;
    const uint32_t i = mdiv(rem, a.mKW);
    const uint32_t j = rem - i * a.kw;
    boff[e] = 4u * ((g * a.Cg + c) * (uint32_t)a.HW + i * a.dh * a.W + j * a.dw);
    bij[e] = MODE == 2 ? i * a.kw + j : ((i * a.dh) << 16) | (j * a.dw);  // tap index, or packed displacement
  }

  const uint32_t c_begin = split * (uint32_t)a.cols_per_split;
  uint32_t c_end = c_begin + (uint32_t)a.cols_per_split;
  if (c_end > (uint32_t)a.ncols) c_end = (uint32_t)a.ncols;
  const int nchunks = c_begin < c_end ? (int)((c_end - c_begin + BK - 1) / BK) : 0;

  M::Acc acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < M::NR; ++r) acc[i][j][r] = 0.f;

  // Both blobs as raw buffer resources: a lane whose column is past the split, or whose tap falls
  // outside the image, presents the buffer size as its offset and the hardware range check
  // returns 0 for it (no branch, no mask to keep).
  const __amdgpu_buffer_rsrc_t dy_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.dy), 0, (int)a.dy_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t x_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.x), 0, (int)a.x_bytes, 0x00020000);

  float ra[A_PER], rb[B_PER];

  // Per-lane state of the column (n, oh, ow) this lane loads in the chunk being fetched.  Elements
  // that must read as zero get an offset at or beyond the blob size (hardware range check returns
  // 0): a column past the split puts 2^31 into both bases; an x tap in the padding either selects
  // the blob size after two compares (MODE 1) or adds bit t of the column's invalid-tap mask,
  // shifted to 2^31 (MODE 2; the mask is the outer product of a row-range and a column-range mask).
  uint32_t dybase = 0, xbase = 0, inv = 0;
  int ih0 = 0, iw0 = 0;
  bool colok = false;
  const int TH = a.khw / a.kw;
  uint32_t row_bits = 0;  // bit i*kw for every tap row i
  if (MODE == 2)
    for (int i = 0; i < TH; ++i) row_bits |= 1u << (i * a.kw);
  auto col_state = [&](int chunk) {
    const uint32_t col = c_begin + chunk * BK + kc;
    colok = col < c_end;
    const uint32_t n = mdiv(col, a.mP);
    const uint32_t pix = col - n * a.P;
    const uint32_t oh = mdiv(pix, a.mPW);
    const uint32_t ow = pix - oh * a.PW;
    ih0 = (int)oh * a.sh - a.ph;
    iw0 = (int)ow * a.sw - a.pw;
    dybase = (colok || MODE == 1) ? 4u * ((n * a.Ktot + g * a.Kg) * (uint32_t)a.P + pix) : 0x80000000u;
    xbase = 4u * (uint32_t)((int)(n * (uint32_t)(a.C * a.HW)) + ih0 * a.W + iw0);
    if (MODE == 0) {
      if (!colok) xbase = 0x80000000u;
    } else if (MODE == 1) {
      if (!colok) ih0 = -(1 << 28);  // fails every bounds test
    } else {
      // taps (i, j) inside the image: i in [lo_i, hi_i), j in [lo_j, hi_j).  The mask over tap index
      // i*kw + j is (bits lo_j..hi_j-1) times (bits i*kw for the valid i): the shifted copies of the
      // column mask do not overlap, so one multiply builds the outer product.
      int lo = -ih0, hi = a.H - ih0;
      lo = lo < 0 ? 0 : (lo > TH ? TH : lo);
      hi = hi < lo ? lo : (hi > TH ? TH : hi);
      const uint32_t rows = row_bits & ((1u << (hi * a.kw)) - (1u << (lo * a.kw)));
      lo = -iw0, hi = a.W - iw0;
      lo = lo < 0 ? 0 : (lo > a.kw ? a.kw : lo);
      hi = hi < lo ? lo : (hi > a.kw ? a.kw : hi);
      const uint32_t colm = (1u << hi) - (1u << lo);
      inv = colok ? ~(colm * rows) : ~0u;
    }
  };
  // DMA: load e of wave wv fills the row pair 4e + wv of the operand's tile in buffer `buf`
  // (rows 8e + 2wv and 8e + 2wv + 1 = rslot + 8e of the two half waves), lane l the l-th word.
  auto load_a = [&](int e, int buf = 0) {
    uint32_t off = dybase + aoff[e];
    if (MODE == 1) off = colok ? off : a.dy_bytes;  // blobs of 2^31 bytes and more: explicit select
    if (DMA)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(dy_rsrc, (LdsPtr)(smem + buf * C::STAGE + (4 * e + wv) * C::PAIR), 4, off,
                                               0, 0, 0);
    else
      ra[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(dy_rsrc, off, 0, 0));
  };
  auto load_b = [&](int e, int buf = 0) {
    uint32_t off = xbase + boff[e];
    if (MODE == 1) {
      const int ih = ih0 + (int)(bij[e] >> 16), iw = iw0 + (int)(bij[e] & 0xffffu);
      const bool ok = ((uint32_t)ih < (uint32_t)a.H) & ((uint32_t)iw < (uint32_t)a.W);
      off = ok ? off : a.x_bytes;
    } else if (MODE == 2) {
      off += __builtin_amdgcn_ubfe(inv, bij[e], 1u) << 31;
    }
    if (DMA)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          x_rsrc, (LdsPtr)(smem + buf * C::STAGE + C::A_FLOATS + (4 * e + wv) * C::PAIR), 4, off, 0, 0, 0);
    else
      rb[e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(x_rsrc, off, 0, 0));
  };
  auto store_a = [&](int buf, int e) { smem[buf * C::STAGE + (rslot + 8 * e) * LDK + kc] = ra[e]; };
  auto store_b = [&](int buf, int e) { smem[buf * C::STAGE + BM * LDK + (rslot + 8 * e) * LDK + kc] = rb[e]; };

  // Software pipeline, three chunks deep (see the correlation kernel): chunk ch is multiplied out
  // of one LDS buffer while the registers holding chunk ch+1 are written to the other buffer and
  // reloaded with chunk ch+2, one or two elements per k step, in the shadow of the MFMAs.
  constexpr int NKS = BK / 2;  // MFMA k steps per chunk; four of them share one 16-byte operand read
  constexpr int NSS = BK / 8;
  const float* opA = smem + C::row_off(wm * MB * 32 + (lane & 31)) + (lane >> 5) * 4;
  const float* opB = smem + C::A_FLOATS + C::row_off(wn * NB * 32 + (lane & 31)) + (lane >> 5) * 4;
  constexpr int BLK = C::row_off(32);  // floats between 32-row blocks
  // Bias gradient from the same read of dy: a wave adds up the dy operands it reads for its MFMAs --
  // lanes l and l + 32 together read every element of row l of a chunk, exactly once.  The work is
  // shared out: every column tile of a split stages the same dy rows, and so do the WN waves of a
  // workgroup that own one row block, so wave wn of column tile n_tile takes the chunks ch with
  // ch % (n_tiles*WN) == n_tile*WN + wn.  The WN waves are added through LDS at the end (in wave
  // order) and the reduce kernel adds the n_tiles shares.  Columns past the split read as zero; rows
  // past the matrix edge are never stored.
  const bool row_sums = a.bias_part != nullptr;
  const int chunk_step = a.n_tiles * WN;
  int my_chunk = (int)n_tile * WN + wn;  // the next chunk whose dy tile this wave sums
  float bsum[MB];
#pragma unroll
  for (int i = 0; i < MB; ++i) bsum[i] = 0.f;
  if (nchunks > 0) {
    col_state(0);
#pragma unroll
    for (int e = 0; e < A_PER; ++e) load_a(e);
#pragma unroll
    for (int e = 0; e < B_PER; ++e) load_b(e);
    if (!DMA) {
#pragma unroll
      for (int e = 0; e < A_PER; ++e) store_a(0, e);
#pragma unroll
      for (int e = 0; e < B_PER; ++e) store_b(0, e);
      col_state(nchunks > 1 ? 1 : 0);
#pragma unroll
      for (int e = 0; e < A_PER; ++e) load_a(e);
#pragma unroll
      for (int e = 0; e < B_PER; ++e) load_b(e);
    } else {
      __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's words of chunk 0 are in LDS
    }
  }
  __syncthreads();
  for (int ch = 0; ch < nchunks; ++ch) {
    const int cur = ch & 1, nxt = cur ^ 1;
    const float* sA = opA + cur * C::STAGE;
    const float* sB = opB + cur * C::STAGE;
    f32x4 av[2][MB], bv[2][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i) av[0][i] = *reinterpret_cast<const f32x4*>(sA + i * BLK);
#pragma unroll
    for (int j = 0; j < NB; ++j) bv[0][j] = *reinterpret_cast<const f32x4*>(sB + j * BLK);
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      const int ss = ks / 4, u = ks % 4;
      if (u == 0 && ss + 1 < NSS) {  // operands of the next group of four steps
#pragma unroll
        for (int i = 0; i < MB; ++i)
          av[(ss + 1) & 1][i] = *reinterpret_cast<const f32x4*>(sA + i * BLK + (ss + 1) * 8);
#pragma unroll
        for (int j = 0; j < NB; ++j)
          bv[(ss + 1) & 1][j] = *reinterpret_cast<const f32x4*>(sB + j * BLK + (ss + 1) * 8);
      }
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) M::run(av[ss & 1][i][u], bv[ss & 1][j][u], acc[i][j]);
      if (u == 3 && row_sums && ch == my_chunk) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
          bsum[i] += (av[ss & 1][i][0] + av[ss & 1][i][1]) + (av[ss & 1][i][2] + av[ss & 1][i][3]);
        if (ss == NSS - 1) my_chunk += chunk_step;
      }
      if (DMA) {
        // this step's share of the loads of chunk ch+1, all issued in the first half of the chunk so
        // that they have the second half to land (past the last chunk they repeat it: nobody reads them)
        constexpr int HALF = NKS / 2;
        if (ks == 0) col_state(ch + 1 < nchunks ? ch + 1 : nchunks - 1);
#pragma unroll
        for (int e = 0; e < A_PER; ++e)
          if (e * HALF / A_PER == ks) load_a(e, nxt);
#pragma unroll
        for (int e = 0; e < B_PER; ++e)
          if (e * HALF / B_PER == ks) load_b(e, nxt);
      } else {
        // this step's share of the staging work: registers of chunk ch+1 go to LDS first ...
#pragma unroll
        for (int e = 0; e < A_PER; ++e)
          if (e * NKS / A_PER == ks) store_a(nxt, e);
#pragma unroll
        for (int e = 0; e < B_PER; ++e)
          if (e * NKS / B_PER == ks) store_b(nxt, e);
        // ... then are reloaded with chunk ch+2 (column state switches once all stores are queued)
        if (ks == 0) col_state(ch + 2 < nchunks ? ch + 2 : nchunks - 1);
#pragma unroll
        for (int e = 0; e < A_PER; ++e)
          if (e * NKS / A_PER == ks) load_a(e);
#pragma unroll
        for (int e = 0; e < B_PER; ++e)
          if (e * NKS / B_PER == ks) load_b(e);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (DMA) __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's words of chunk ch+1 are in LDS
    __syncthreads();
  }

  if (row_sums) {  // uniform over the grid; the pipeline buffers are free after the loop's last barrier
    float* red = smem;  // [WN][BM]
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      const float total = bsum[i] + __shfl_xor(bsum[i], 32);
      if (lane < 32) red[wn * BM + (wm * MB + i) * 32 + lane] = total;
    }
    __syncthreads();
    if (wn == 0 && lane < 32) {
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        const int row = (wm * MB + i) * 32 + lane;
        float total = red[row];
#pragma unroll
        for (int v = 1; v < WN; ++v) total += red[v * BM + row];
        const uint32_t k = m_tile * BM + (uint32_t)row;
        if (k < (uint32_t)a.Kg) a.bias_part[((size_t)split * a.n_tiles + n_tile) * a.Ktot + g * a.Kg + k] = total;
      }
    }
  }

  // partial tile -> workspace [split][g][k][nn]
  float* dst = a.part + (size_t)split * a.part_stride + (size_t)g * ((size_t)a.Kg * a.Kred);
  const uint64_t slice_bytes = 4ull * (uint64_t)a.Kg * (uint64_t)a.Kred;
  if (slice_bytes <= (1ull << 30)) {
    // Byte offsets per row and per column with out-of-range values for rows and columns past the
    // matrix edge (2^31 and 2^30: any sum with one of them lies beyond the slice); the range check
    // of the buffer store drops those elements.
    const __amdgpu_buffer_rsrc_t out_rsrc = __builtin_amdgcn_make_buffer_rsrc(dst, 0, (int)slice_bytes, 0x00020000);
    uint32_t co[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const uint32_t nn = n_tile * BN + (wn * NB + j) * 32 + (lane & 31);
      co[j] = nn < (uint32_t)a.Kred ? 4u * nn : 0x40000000u;
    }
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int r = 0; r < M::NR; ++r) {
        const uint32_t k = m_tile * BM + (wm * MB + i) * 32 + M::row(r, lane);
        const uint32_t ro = k < (uint32_t)a.Kg ? 4u * k * (uint32_t)a.Kred : 0x80000000u;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          const float v = acc[i][j][r];  // a named float: a bit cast applied to the vector element itself stored zeros
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), out_rsrc, ro + co[j], 0, 0);
        }
      }
    return;
  }
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const uint32_t nn = n_tile * BN + (wn * NB + j) * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int r = 0; r < M::NR; ++r) {
        const uint32_t k = m_tile * BM + (wm * MB + i) * 32 + M::row(r, lane);
        if (k < (uint32_t)a.Kg && nn < (uint32_t)a.Kred) dst[(size_t)k * a.Kred + nn] = acc[i][j][r];
      }
  }
}

template <int MB, int NB, int WM, int WN, int MODE, bool DMA>
int launch_wgrad_m(const WgradArgs& a, hipStream_t s) {
  using C = WgCfg<MB, NB, WM, WN, DMA>;
  static LdsOptIn opt_in;  // more than 64 KB of LDS needs an explicit opt-in, once per process
  if (const int e = lds_opt_in(opt_in, &wgrad_kernel<MB, NB, WM, WN, MODE, DMA>, C::SMEM_BYTES)) return e;
  const uint32_t blocks = (uint32_t)a.G * a.S * a.m_tiles * a.n_tiles;
  hipLaunchKernelGGL((wgrad_kernel<MB, NB, WM, WN, MODE, DMA>), dim3(blocks), dim3(kThreads), C::SMEM_BYTES, s, a);
  return (int)hipGetLastError();
}

template <int MB, int NB, int WM, int WN, bool DMA>
int launch_wgrad_t(const WgradArgs& a, hipStream_t s) {
  if (a.bounds_mode == 0) return launch_wgrad_m<MB, NB, WM, WN, 0, DMA>(a, s);
  if (a.bounds_mode == 2) return launch_wgrad_m<MB, NB, WM, WN, 2, DMA>(a, s);
  return launch_wgrad_m<MB, NB, WM, WN, 1, DMA>(a, s);
}

// dst = beta*dst + sum_s part[s] (+ bias, ReLU).  A block owns 64*V consecutive elements (V = 4 with
// 16-byte accesses when the element count is a multiple of four and the blobs are 16-byte aligned,
// else 1); its four waves each add a contiguous quarter of the splits (four independent chains per
// lane), and the four quarter sums are combined in a fixed order, so the result does not depend on
// scheduling.
template <int V>
__global__ __launch_bounds__(256) void reduce_kernel(const ReduceArgs a) {
  struct alignas(4 * V) Vec {
    float v[V];
  };
  __shared__ Vec quarter[4][64];
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  // workgroups past those of the first reduction take the second one (uniform per workgroup)
  const int blocks1 = (a.count / V + 63) / 64;
  const bool second = (int)blockIdx.x >= blocks1;
  const int i = (((int)blockIdx.x - (second ? blocks1 : 0)) * 64 + lane) * V;
  const int S = second ? a.S2 : a.S;
  const int per = (S + 3) / 4;
  const int s0 = q * per;
  int s1 = s0 + per;
  if (s1 > S) s1 = S;
  Vec acc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int e = 0; e < V; ++e) acc[c].v[e] = 0.f;
  constexpr int U = V == 1 ? 16 : 4;  // loads in flight per lane: a long run of slices is latency-bound
  const int total = second ? a.count2 : a.count;
  const size_t stride = second ? (size_t)a.count2 : a.stride ? (size_t)a.stride : (size_t)a.count;
  if (i < total) {
    const float* src = (second ? a.part2 : a.part) + i;
    int k = s0;
    for (; k + U - 1 < s1; k += U) {
      Vec x[U];
#pragma unroll
      for (int c = 0; c < U; ++c) x[c] = *reinterpret_cast<const Vec*>(src + (size_t)(k + c) * stride);
#pragma unroll
      for (int c = 0; c < U; ++c)
#pragma unroll
        for (int e = 0; e < V; ++e) acc[c & 3].v[e] += x[c].v[e];
    }
    for (; k + 3 < s1; k += 4) {
      Vec x[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) x[c] = *reinterpret_cast<const Vec*>(src + (size_t)(k + c) * stride);
#pragma unroll
      for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int e = 0; e < V; ++e) acc[c].v[e] += x[c].v[e];
    }
    for (; k < s1; ++k) {
      const Vec x = *reinterpret_cast<const Vec*>(src + (size_t)k * stride);
#pragma unroll
      for (int e = 0; e < V; ++e) acc[0].v[e] += x.v[e];
    }
  }
  Vec sum;
#pragma unroll
  for (int e = 0; e < V; ++e) sum.v[e] = (acc[0].v[e] + acc[1].v[e]) + (acc[2].v[e] + acc[3].v[e]);
  quarter[q][lane] = sum;
  __syncthreads();
  if (q == 0 && i < total) {
    Vec out, old;
    float* const dst = (second ? a.dst2 : a.dst) + i;
    const bool first = !second;
    if (a.beta != 0.f) old = *reinterpret_cast<const Vec*>(dst);
#pragma unroll
    for (int e = 0; e < V; ++e) {
      float s = (quarter[0][lane].v[e] + quarter[1][lane].v[e]) + (quarter[2][lane].v[e] + quarter[3][lane].v[e]);
      if (a.bias && first) {
        const uint32_t c = mdiv((uint32_t)(i + e), a.mChanElems);
        s += a.bias[c - mdiv(c, a.mChannels) * a.channels];
      }
      if (a.beta != 0.f) s += a.beta * old.v[e];
      if (a.relu && first) s = s > 0.f ? s : 0.f;
      out.v[e] = s;
    }
    *reinterpret_cast<Vec*>(dst) = out;
  }
}

}  // namespace

void wgrad_tile_shape(int32_t tile, int32_t* bm, int32_t* bn, int32_t* bk) {
  static const int32_t shapes[WGRAD_TILE_COUNT][3] = {
      {128, 128, 32}, {96, 128, 32}, {64, 128, 32}, {32, 128, 32}, {128, 64, 32}};
  *bm = shapes[tile][0];
  *bn = shapes[tile][1];
  *bk = shapes[tile][2];
}

const char* wgrad_tile_name(int32_t tile) {
  static const char* names[WGRAD_TILE_COUNT] = {"wgrad_m32_128x128x32", "wgrad_m32_96x128x32", "wgrad_m32_64x128x32",
                                                "wgrad_m32_32x128x32", "wgrad_m32_128x64x32"};
  return names[tile];
}

int launch_wgrad(int32_t tile, const WgradArgs& a, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  // Loads that write LDS themselves pay on the square tile (5.b, 5.c backward filter 1.5 % faster); the
  // 96-row tile with its short splits and stride-4 gather is 1 % slower with them, the narrow tiles
  // show no difference.
  switch (tile) {
    case WGRAD_128x128: return launch_wgrad_t<2, 2, 2, 2, true>(a, s);
    case WGRAD_96x128:  return launch_wgrad_t<3, 1, 1, 4, false>(a, s);
    case WGRAD_64x128:  return launch_wgrad_t<2, 1, 1, 4, false>(a, s);
    case WGRAD_32x128:  return launch_wgrad_t<1, 1, 1, 4, false>(a, s);
    case WGRAD_128x64:  return launch_wgrad_t<2, 1, 2, 2, false>(a, s);
    default: return (int)hipErrorInvalidValue;
  }
}

int launch_reduce(const ReduceArgs& a, void* stream) {
  // the four-element form needs enough elements to keep a thousand workgroups busy
  const bool vec = a.count >= (1 << 18) && a.count % 4 == 0 && a.count2 % 4 == 0 && a.stride % 4 == 0 &&
                   ((reinterpret_cast<uintptr_t>(a.part) | reinterpret_cast<uintptr_t>(a.dst) |
                     reinterpret_cast<uintptr_t>(a.part2) | reinterpret_cast<uintptr_t>(a.dst2)) & 15u) == 0;
  if (vec)
    hipLaunchKernelGGL(reduce_kernel<4>, dim3((a.count / 4 + 63) / 64 + (a.count2 / 4 + 63) / 64), dim3(256), 0,
                       (hipStream_t)stream, a);
  else
    hipLaunchKernelGGL(reduce_kernel<1>, dim3((a.count + 63) / 64 + (a.count2 + 63) / 64), dim3(256), 0,
                       (hipStream_t)stream, a);
  return (int)hipGetLastError();
}

}  // namespace mi355conv
