// Tiled forward kernel for 3x3 tropical convolutions in binary16 arithmetic on gfx950: the packed 16-bit VALU path.
//
// Operator: paper Sec. 3.1 layers (iv) / (v) and the Sec. 3.3 compound / parallel combinations, with the numeric
// contract of dtype TCONV_F16: every candidate x + w is one add rounded to binary16, the reductions compare those
// binary16 sums, ties keep the lowest flattened tap k; the combine is evaluated in fp32 from the binary16 extrema and
// rounded to binary16 once.
//
// The scheme is the one of the fp32 tiled kernel (a lane owns 8 consecutive output pixels of a row and a few output
// channels, the extrema stay in registers for the whole K loop, kernel values are wave-uniform scalar operands,
// padding is NaN and never wins, the winner is tracked coarsely in the loop and refined afterwards) with the
// following differences, all of which come from the packed instructions:
//  * The two halves of a register are two OUTPUT CHANNELS: a lane owns 2 channel pairs = 4 channels x 8 pixels.
//    The kernel tensors are first re-laid (a small kernel, into the workspace) as [C_out / 2][K] dwords holding
//    (w[2c][k], w[2c + 1][k]), which scalar loads put into SGPRs: one v_pk_add_f16 adds one x value to two kernel
//    values, one v_pk_max_f16 / v_pk_min_f16 folds two candidates.  Compound mode: 62 instructions per 72 pairs.
//  * x stays packed as loaded, two neighbouring columns per register (one 16-byte load per row and channel for the 8
//    core columns, single 16-bit loads for the halo columns); the packed add picks the half it needs with its
//    operand-select bits, so no instruction is spent on unpacking or broadcasting.  This needs every lane's core
//    columns to start at an even element: W even and an even left margin (dilation - pad_w); other layers run on
//    the generic kernel.
//  * The loop records the input-channel PAIR at which a half of an extremum changed (see the blocks header); the
//    exact tap is the first of the pair's 18 taps, in k order, whose binary16 sum equals the extremum.
//  * Two full sets of x rows and two sets of extrema alternate (the pair loop is unrolled by two): no copies.
#include <stdlib.h>

#include <utility>

#include "tile_common.h"
// after tile_common.h: the blocks header relies on the HIP runtime declarations included there
#include <tile_blocks_f16_gfx950.h>

namespace tconv {
namespace {

using namespace tile;

constexpr int PX = 8;    // output pixels per lane
constexpr int TNP = 2;   // output-channel pairs per lane
constexpr int TN = 2 * TNP;

template <int... Q, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Q...>, F&& f) {
  (f(std::integral_constant<int, Q>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F&&>(f));
}

__device__ __forceinline__ int launder(int v) {  // the compiler forgets the value of a wave-uniform integer
  asm volatile("" : "+s"(v));
  return v;
}

typedef unsigned u4a __attribute__((ext_vector_type(4), aligned(4)));

// 8 consecutive binary16 outputs (bits in the low halves of v) -> memory; pixels q < first_q belong to the
// neighbouring lane.  The row start is 4-byte aligned (W_out and the first column of a segment are even).
__device__ __forceinline__ void store_row16(f16_t* p, const unsigned (&v)[PX], int first_q) {
  if (first_q == 0) {
    u4a a;
    a.x = v[0] | (v[1] << 16); a.y = v[2] | (v[3] << 16); a.z = v[4] | (v[5] << 16); a.w = v[6] | (v[7] << 16);
    *(u4a*)p = a;
  } else {
    unsigned short* ps = (unsigned short*)p;
#pragma unroll
    for (int q = 0; q < PX; ++q)
      if (q >= first_q) ps[q] = (unsigned short)v[q];
  }
}

__device__ __forceinline__ float half_bits_to_float(unsigned b) {
  union { unsigned short u; f16_t h; } c;
  c.u = (unsigned short)b;
  return (float)c.h;
}
__device__ __forceinline__ unsigned float_to_half_bits(float v) {
  union { unsigned short u; f16_t h; } c;
  c.h = (f16_t)v;  // round to nearest even
  return c.u;
}

// wp_*: the re-laid kernel tensors [ceil(C_out / 2)][KP] dwords, KP = 18 * ceil(C_in / 2) (rows padded to whole
// channel pairs), read by the main loop through scalar loads and by the tap recovery through gathers.
template <int MODE, int D, bool PZ>
__global__ __launch_bounds__(WAVES * 64, 2) void fwd_tiled3x3_f16_kernel(
    Params p, const f16_t* __restrict__ x, const unsigned* __restrict__ wp_min, const unsigned* __restrict__ wp_max,
    const float* __restrict__ alpha,
    const float* __restrict__ beta, f16_t* __restrict__ y, f16_t* __restrict__ y_min, f16_t* __restrict__ y_max,
    int32_t* __restrict__ idx_min, int32_t* __restrict__ idx_max, int segs, int n_units, int n_groups, int n_ublocks,
    int xsplit) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr int XRP = 4 + 2 * D;  // registers per x row: D halo, 4 x 2 core columns, D halo
  constexpr unsigned NEG_INF2 = 0xfc00fc00u, POS_INF2 = 0x7c007c00u;

  // ---- which output-channel group (wave-uniform) and which pixel segment (per lane); the 8 XCDs split the work into
  // xsplit parts of the channel blocks times 8 / xsplit parts of the pixel blocks, as in the fp32 kernel
  const int gblocks = (n_groups + WAVES - 1) / WAVES;
  int ublock, gblock;
  {
    const int xcd = (int)(blockIdx.x & 7u), j = (int)(blockIdx.x >> 3);
    const int gb_per = (gblocks + xsplit - 1) / xsplit;
    const int pparts = 8 / xsplit;
    const int ub_per = (n_ublocks + pparts - 1) / pparts;
    const int lu = j / gb_per, lg = j - lu * gb_per;
    ublock = (xcd / xsplit) * ub_per + lu;
    gblock = (xcd & (xsplit - 1)) * gb_per + lg;
    if (lu >= ub_per || ublock >= n_ublocks || gblock >= gblocks) return;  // grid padding; the kernel has no barrier
  }
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int group = gblock * WAVES + wave;
  if (group >= n_groups) return;  // whole wave leaves
  const int co0 = group * TN;
  const int lane = threadIdx.x & 63;
  const int unit_raw = ublock * 64 + lane;
  const bool unit_ok = unit_raw < n_units;
  const int unit = unit_ok ? unit_raw : n_units - 1;  // surplus lanes recompute the last unit, store nothing
  const int seg = unit % segs;
  const int oh = (unit / segs) % p.Ho;
  const int n = unit / (segs * p.Ho);
  const int ow_nom = seg * PX;
  const int ow0 = min(ow_nom, p.Wo - PX);  // the last segment of a row is shifted left (even: W_out is even)
  const int first_q = ow_nom - ow0;

  // ---- channel-independent addressing and padding masks (all byte offsets of binary16 elements)
  const int iw0 = ow0 - p.pw;  // input column of row element 0
  const size_t HW = (size_t)p.H * p.W;
  const rsrc_t xres = make_rsrc(x, (unsigned)((size_t)p.N * p.C_in * HW * 2));
  unsigned roff[3];  // byte offset of the first core column (iw0 + D, even and inside the row) of each clamped row
  unsigned mrow[3];  // identity padding: all-ones where the row is padding; zero padding: all-ones where it is NOT
  int ihc[3];
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int ih = oh - p.ph + i * D;
    mrow[i] = ((ih >= 0 && ih < p.H) != PZ) ? 0u : 0xffffffffu;
    ihc[i] = min(max(ih, 0), p.H - 1);
    roff[i] = (unsigned)(((size_t)n * p.C_in * HW + (size_t)ihc[i] * p.W + (size_t)(iw0 + D)) * 2);
  }
  int hoff[2 * D];
  unsigned mhalo[2 * D];
#pragma unroll
  for (int h = 0; h < 2 * D; ++h) {
    const int o = (h < D) ? h : h + 8;
    const int iw = iw0 + o;
    mhalo[h] = ((iw >= 0 && iw < p.W) != PZ) ? 0u : 0xffffffffu;
    hoff[h] = (min(max(iw, 0), p.W - 1) - (iw0 + D)) * 2;
  }

  // ---- re-laid kernel rows of this wave's channel pairs (wave-uniform)
  const int n_cpairs = (p.C_out + 1) >> 1;
  const int ndu = (p.C_in + 1) >> 1;  // input-channel pairs
  const int KP = 18 * ndu;
  const unsigned* wr_min[TNP];
  const unsigned* wr_max[TNP];
#pragma unroll
  for (int c = 0; c < TNP; ++c) {
    const int cp = min(co0 / 2 + c, n_cpairs - 1);
    wr_min[c] = DO_MIN ? wp_min + (size_t)cp * KP : nullptr;
    wr_max[c] = DO_MAX ? wp_max + (size_t)cp * KP : nullptr;
  }

  // two sets of running extrema (a block reads one and writes the other) and one set of recorded pairs
  unsigned amax[2][TNP][PX], amin[2][TNP][PX], imax[TNP][PX], imin[TNP][PX];
#pragma unroll
  for (int c = 0; c < TNP; ++c)
#pragma unroll
    for (int q = 0; q < PX; ++q) {
      amax[0][c][q] = NEG_INF2; amin[0][c][q] = POS_INF2;
      amax[1][c][q] = NEG_INF2; amin[1][c][q] = POS_INF2;
      imax[c][q] = 0; imin[c][q] = 0;
    }
  const unsigned one2 = 0x00010001u;

  // channel pairs du = 0 .. ndu - 1 (channels 2du, 2du + 1); the loop runs an even number of them: a pair past the
  // end, and the second channel of the last pair when C_in is odd, are all NaN
  auto chan_soff = [&](int c) -> unsigned { return (unsigned)((size_t)min(c, p.C_in - 1) * HW * 2); };
  auto issue_rows = [&](unsigned (&xs)[6][XRP], int du) {
#pragma unroll
    for (int sl = 0; sl < 6; ++sl) {
      const unsigned soff = chan_soff(2 * du + sl / 3);
      const unsigned ro = roff[sl % 3];
#pragma unroll
      for (int h = 0; h < D; ++h)
        xs[sl][h] = (unsigned)__builtin_amdgcn_raw_buffer_load_b16(xres, ro + (unsigned)hoff[h], soff, 0);
      const u4v v = __builtin_amdgcn_raw_buffer_load_b128(xres, ro, soff, 0);
      xs[sl][D] = v.x; xs[sl][D + 1] = v.y; xs[sl][D + 2] = v.z; xs[sl][D + 3] = v.w;
#pragma unroll
      for (int h = 0; h < D; ++h)
        xs[sl][D + 4 + h] = (unsigned)__builtin_amdgcn_raw_buffer_load_b16(xres, ro + (unsigned)hoff[D + h], soff, 0);
    }
  };
  // padding -> NaN (identity padding) or +0 (zero padding); channels past C_in -> NaN always
  auto mask_rows = [&](unsigned (&xs)[6][XRP], int du) {
#pragma unroll
    for (int sl = 0; sl < 6; ++sl) {
      const unsigned vB = (2 * du + sl / 3 < p.C_in) ? 0u : 0xffffffffu;
      const unsigned mr = PZ ? mrow[sl % 3] : (mrow[sl % 3] | vB);
#pragma unroll
      for (int r = 0; r < XRP; ++r) {
        unsigned m = mr;
        if (r < D) m = PZ ? (m & mhalo[r]) : (m | mhalo[r]);
        if (r >= D + 4) m = PZ ? (m & mhalo[r - 4]) : (m | mhalo[r - 4]);
        xs[sl][r] = PZ ? ((xs[sl][r] & m) | vB) : (xs[sl][r] | m);
      }
    }
  };
  auto load_w = [&](unsigned (&wv)[18], const unsigned* row, int du) {
    const unsigned* pw_ = row + launder(min(du, ndu - 1) * 18);  // a pair past the end re-reads the last one
#pragma unroll
    for (int t = 0; t < 18; ++t) wv[t] = pw_[t];
  };
  // kernel rows of a pair in the order they are used: per channel pair c the max row, then the min row (compound:
  // the one shared row)
  constexpr int NR = (MODE == TCONV_PARALLEL) ? 2 * TNP : TNP;
  auto row_of = [&](int r) -> const unsigned* {
    if (MODE == TCONV_PARALLEL) return (r & 1) ? wr_min[r >> 1] : wr_max[r >> 1];
    return DO_MAX ? wr_max[r] : wr_min[r];
  };
  // one channel pair: every pixel and output-channel pair of the lane, from extrema set SRC into set 1 - SRC
  auto do_pair = [&](auto src_tag, unsigned (&xs)[6][XRP], int du, unsigned (&wc)[18]) {
    constexpr int SRC = decltype(src_tag)::value;
    const unsigned tid = (unsigned)du | ((unsigned)du << 16);
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      // the kernel values of the next row to run (next row of this pair, or the first row of the next pair) are
      // fetched while this row's blocks run
      unsigned wn[18];
      load_w(wn, row_of((r + 1) % NR), r + 1 < NR ? du : du + 1);
      const int c = (MODE == TCONV_PARALLEL) ? (r >> 1) : r;
      static_for<PX>([&](auto qt) {
        constexpr int Q = decltype(qt)::value;
        if constexpr (MODE == TCONV_COMPOUND) {
          f16blk::blk_both<D, Q>(amax[1 - SRC][c][Q], amin[1 - SRC][c][Q], amax[SRC][c][Q], amin[SRC][c][Q],
                                 imax[c][Q], imin[c][Q], xs, wc, tid, one2);
        } else if constexpr (MODE == TCONV_PARALLEL) {
          if (r & 1) f16blk::blk_min<D, Q>(amin[1 - SRC][c][Q], amin[SRC][c][Q], imin[c][Q], xs, wc, tid, one2);
          else f16blk::blk_max<D, Q>(amax[1 - SRC][c][Q], amax[SRC][c][Q], imax[c][Q], xs, wc, tid, one2);
        } else if constexpr (MODE == TCONV_MAX) {
          f16blk::blk_max<D, Q>(amax[1 - SRC][c][Q], amax[SRC][c][Q], imax[c][Q], xs, wc, tid, one2);
        } else {
          f16blk::blk_min<D, Q>(amin[1 - SRC][c][Q], amin[SRC][c][Q], imin[c][Q], xs, wc, tid, one2);
        }
      });
#pragma unroll
      for (int t = 0; t < 18; ++t) wc[t] = wn[t];
    }
  };

  {
    unsigned xs0[6][XRP], xs1[6][XRP];
    unsigned wc[18];
    issue_rows(xs0, 0);
    load_w(wc, row_of(0), 0);
    for (int du = 0; du < ndu; du += 2) {
      issue_rows(xs1, du + 1);
      mask_rows(xs0, du);
      do_pair(std::integral_constant<int, 0>{}, xs0, du, wc);
      issue_rows(xs0, du + 2);
      mask_rows(xs1, du + 1);
      do_pair(std::integral_constant<int, 1>{}, xs1, du + 1, wc);
    }
  }
  // the extrema are in set 0 again

  // ---- epilogue: exact tap of every extremum, combine, store.
  // An output's winner is searched among the 18 taps of its recorded input-channel pair: the 18 kernel-value dwords
  // of the pair (five wide loads from the re-laid tensor; the output channel is a compile-time half), the core
  // columns of its six x rows (one 16-byte load each: they start at an even element) and, for the first and last D
  // pixels of the lane, the halo columns.  Each candidate is one packed add whose operand-select bits pick the halves
  // and leave the sum in the low half; walking the taps downwards keeps the lowest matching k.
  const int first_qs = unit_ok ? first_q : PX;  // surplus lanes store nothing
  const rsrc_t wpres_min = make_rsrc(DO_MIN ? wp_min : wp_max, (unsigned)((size_t)n_cpairs * KP * 4));
  const rsrc_t wpres_max = make_rsrc(DO_MAX ? wp_max : wp_min, (unsigned)((size_t)n_cpairs * KP * 4));
  const unsigned HW2 = (unsigned)(HW * 2);  // < 2^24 (checked on the host)
  bool rowok[3], halook[2 * D];
#pragma unroll
  for (int i = 0; i < 3; ++i) rowok[i] = PZ ? (mrow[i] != 0u) : (mrow[i] == 0u);
#pragma unroll
  for (int h = 0; h < 2 * D; ++h) halook[h] = PZ ? (mhalo[h] != 0u) : (mhalo[h] == 0u);
  auto refine = [&](auto qt, auto hht, rsrc_t wpres, unsigned cp_soff, unsigned du, unsigned best) -> int {
    constexpr int Q = decltype(qt)::value, HH = decltype(hht)::value;
    unsigned wv[18];
    {
      const unsigned wb = __umul24(du, 72u);
      const u4v a0 = __builtin_amdgcn_raw_buffer_load_b128(wpres, wb, cp_soff, 0);
      const u4v a1 = __builtin_amdgcn_raw_buffer_load_b128(wpres, wb + 16u, cp_soff, 0);
      const u4v a2 = __builtin_amdgcn_raw_buffer_load_b128(wpres, wb + 32u, cp_soff, 0);
      const u4v a3 = __builtin_amdgcn_raw_buffer_load_b128(wpres, wb + 48u, cp_soff, 0);
      const u2v a4 = __builtin_amdgcn_raw_buffer_load_b64(wpres, wb + 64u, cp_soff, 0);
      wv[0] = a0.x; wv[1] = a0.y; wv[2] = a0.z; wv[3] = a0.w; wv[4] = a1.x; wv[5] = a1.y; wv[6] = a1.z; wv[7] = a1.w;
      wv[8] = a2.x; wv[9] = a2.y; wv[10] = a2.z; wv[11] = a2.w; wv[12] = a3.x; wv[13] = a3.y; wv[14] = a3.z;
      wv[15] = a3.w; wv[16] = a4.x; wv[17] = a4.y;
    }
    unsigned xr[6][XRP];  // the rows in the register layout of the main loop
    bool cvalid[2];
#pragma unroll
    for (int ch = 0; ch < 2; ++ch) {
      const int c = 2 * (int)du + ch;
      cvalid[ch] = c < p.C_in;
      const unsigned choff = __umul24((unsigned)min(c, p.C_in - 1), HW2);
#pragma unroll
      for (int i = 0; i < 3; ++i) {
        const unsigned base = roff[i] + choff;
        const u4v v = __builtin_amdgcn_raw_buffer_load_b128(xres, base, 0, 0);
        xr[ch * 3 + i][D] = v.x; xr[ch * 3 + i][D + 1] = v.y; xr[ch * 3 + i][D + 2] = v.z; xr[ch * 3 + i][D + 3] = v.w;
#pragma unroll
        for (int h = 0; h < 2 * D; ++h) {
          // halo column h is read by this pixel iff one of its taps falls on row element e = h (left) or h + 8 (right)
          const int e = h < D ? h : h + 8;
          const bool used = (e == Q) || (e == Q + D) || (e == Q + 2 * D);
          const int r = h < D ? h : h + 4;
          if (used) {
            unsigned hv = (unsigned)__builtin_amdgcn_raw_buffer_load_b16(xres, base + (unsigned)hoff[h], 0, 0);
            if (PZ && !halook[h]) hv = 0u;
            xr[ch * 3 + i][r] = hv;
          } else {
            xr[ch * 3 + i][r] = 0u;
          }
        }
        if (PZ && !rowok[i]) {
#pragma unroll
          for (int r = 0; r < XRP; ++r) xr[ch * 3 + i][r] = 0u;
        }
      }
    }
    int r = 0;
    static_for<18>([&](auto tt) {
      constexpr int t = 17 - decltype(tt)::value;  // downwards
      constexpr int ch = t / 9, i = (t % 9) / 3, j = t % 3;
      constexpr int e = Q + j * D;
      constexpr int reg = f16blk::xreg(D, e), hx = f16blk::xhalf(D, e);
      constexpr bool halo = e < D || e >= D + 8;
      constexpr int h = e < D ? e : e - 8;  // halo number when halo
      unsigned sum;
      asm("v_pk_add_f16 %0, %1, %2 op_sel:[%3,%4] op_sel_hi:[%3,%4]"
          : "=v"(sum) : "v"(xr[ch * 3 + i][reg]), "v"(wv[t]), "n"(hx), "n"(HH));
      bool ok = cvalid[ch];
      if (!PZ) {
        ok = ok && rowok[i];
        if (halo) ok = ok && halook[halo ? h : 0];
      }
      r = (ok && (unsigned short)sum == (unsigned short)best) ? t : r;
    });
    return (int)__umul24(du, 18u) + r;
  };
  const size_t plane = (size_t)p.Ho * p.Wo;
  static_for<TN>([&](auto cht) {
    constexpr int c = decltype(cht)::value / 2, hh = decltype(cht)::value % 2;
    const int co = co0 + 2 * c + hh;
    if (co < p.C_out) {  // wave-uniform
      const unsigned cp_soff = (unsigned)((size_t)(co0 / 2 + c) * KP * 4);
      const size_t ob = ((size_t)n * p.C_out + co) * plane + (size_t)oh * p.Wo + ow0;
      float ca = 1.f, cb = 1.f;
      if (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL) {
        if (alpha) ca = alpha[co];
        if (beta) cb = beta[co];
      }
      unsigned vmin[PX], vmax[PX], out[PX];
      int ridx[PX];
      if (DO_MIN) {
        static_for<PX>([&](auto qt) {
          constexpr int q = decltype(qt)::value;
          vmin[q] = (amin[0][c][q] >> (16 * hh)) & 0xffffu;
          ridx[q] = refine(qt, std::integral_constant<int, hh>{}, wpres_min, cp_soff,
                           (imin[c][q] >> (16 * hh)) & 0xffffu, vmin[q]);
        });
        store_row<PX>(idx_min + ob, ridx, first_qs);
        if (y_min) store_row16(y_min + ob, vmin, first_qs);
      }
      if (DO_MAX) {
        static_for<PX>([&](auto qt) {
          constexpr int q = decltype(qt)::value;
          vmax[q] = (amax[0][c][q] >> (16 * hh)) & 0xffffu;
          ridx[q] = refine(qt, std::integral_constant<int, hh>{}, wpres_max, cp_soff,
                           (imax[c][q] >> (16 * hh)) & 0xffffu, vmax[q]);
        });
        store_row<PX>(idx_max + ob, ridx, first_qs);
        if (y_max) store_row16(y_max + ob, vmax, first_qs);
      }
#pragma unroll
      for (int q = 0; q < PX; ++q) {
        if (!DO_MIN) out[q] = vmax[q];
        else if (!DO_MAX) out[q] = vmin[q];
        else out[q] = float_to_half_bits(combine(ca, half_bits_to_float(vmin[q]), cb, half_bits_to_float(vmax[q])));
      }
      store_row16(y + ob, out, first_qs);
    }
  });
}

// (w[2c][k], w[2c + 1][k]) -> dword [c][k] of a row of KP >= K dwords (the tail is zero); an odd C_out repeats its
// last channel in the upper half
__global__ __launch_bounds__(256) void relay_pairs_kernel(const unsigned short* __restrict__ w,
                                                          unsigned* __restrict__ wp, int C_out, int K, int KP) {
  const int n_cpairs = (C_out + 1) >> 1;
  const size_t total = (size_t)n_cpairs * KP, stride = (size_t)gridDim.x * blockDim.x;
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
    const size_t cp = e / (size_t)KP, k = e - cp * (size_t)KP;
    const size_t c0 = 2 * cp, c1 = min(2 * cp + 1, (size_t)C_out - 1);
    wp[e] = k < (size_t)K ? ((unsigned)w[c0 * K + k] | ((unsigned)w[c1 * K + k] << 16)) : 0u;
  }
}

size_t relaid_dwords(const Params& p) { return (size_t)((p.C_out + 1) / 2) * 18 * ((p.C_in + 1) / 2); }

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

template <int MODE, int D, bool PZ>
hipError_t launch_k(const Params& p, const FwdArgs& a, const unsigned* wp_min, const unsigned* wp_max,
                    hipStream_t s) {
  const int segs = (p.Wo + PX - 1) / PX;
  const long long n_units = (long long)p.N * p.Ho * segs;
  const int n_groups = (p.C_out + TN - 1) / TN;
  const long long ublocks = (n_units + 63) / 64;
  const long long gblocks = (n_groups + WAVES - 1) / WAVES;
  // the XCDs split the work as in the fp32 kernel: parts of the (re-laid) kernel tensors of at most 1.5 MB
  const long long w_bytes = (long long)relaid_dwords(p) * 4 * (MODE == TCONV_PARALLEL ? 2 : 1);
  int xsplit = 1;
  while (xsplit < 8 && w_bytes / xsplit > 1536LL * 1024 && 2 * xsplit <= gblocks) xsplit *= 2;
  const long long gb_per = (gblocks + xsplit - 1) / xsplit, ub_per = (ublocks + 8 / xsplit - 1) / (8 / xsplit);
  const long long grid = 8 * gb_per * ub_per;
  if (grid > 0x7ffffff0LL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((fwd_tiled3x3_f16_kernel<MODE, D, PZ>), dim3((unsigned)grid), dim3(WAVES * 64), 0, s, p,
                     (const f16_t*)a.x, wp_min, wp_max, a.alpha, a.beta,
                     (f16_t*)a.y, (f16_t*)a.y_min, (f16_t*)a.y_max, a.idx_min, a.idx_max, segs, (int)n_units,
                     n_groups, (int)ublocks, xsplit);
  return hipGetLastError();
}

template <int MODE>
hipError_t launch_m(const Params& p, const FwdArgs& a, const unsigned* wp_min, const unsigned* wp_max,
                    hipStream_t s) {
  if (p.dh == 1)
    return p.pad_zero ? launch_k<MODE, 1, true>(p, a, wp_min, wp_max, s)
                      : launch_k<MODE, 1, false>(p, a, wp_min, wp_max, s);
  return p.pad_zero ? launch_k<MODE, 2, true>(p, a, wp_min, wp_max, s)
                    : launch_k<MODE, 2, false>(p, a, wp_min, wp_max, s);
}

}  // namespace

// 3x3 kernels at stride 1 with dilation 1 or 2 on both axes, the four full-window modes, W even and an even left
// margin dilation - pad_w >= 0 (every lane's core columns then start at an even element of x and are never
// padding), at least one full pixel segment per output row, tensors addressable with 32-bit byte offsets.
bool forward_tiled3x3_f16_supported(const Params& p, int dtype) {
  if (dtype != TCONV_F16 || p.mode > TCONV_PARALLEL) return false;
  if (p.KH != 3 || p.KW != 3 || p.sh != 1 || p.sw != 1) return false;
  if (p.dh != p.dw || (p.dh != 1 && p.dh != 2)) return false;
  if (p.pw > p.dw || ((p.dw - p.pw) & 1) || (p.W & 1)) return false;
  if (p.Wo < PX || p.W < 2 * p.dw + 1) return false;
  if (p.C_in > 2 * 65535) return false;  // pair numbers are recorded as 16-bit values
  if ((size_t)p.H * p.W * 2 >= (1u << 24)) return false;  // channel offsets come from 24-bit multiplies
  if ((size_t)p.N * p.C_in * p.H * p.W * 2 >= 0xfffff000ull) return false;
  if ((size_t)(p.C_out + 1) * (p.K + 9) * 4 >= 0xfffff000ull) return false;
  return true;
}

// the re-laid kernel tensors
size_t forward_tiled3x3_f16_workspace(const Params& p) {
  return align256(relaid_dwords(p) * 4) * (p.mode == TCONV_PARALLEL ? 2 : 1);
}

hipError_t launch_forward_tiled3x3_f16(const Params& p, const FwdArgs& a, void* workspace, hipStream_t s) {
  const size_t n_pairs = relaid_dwords(p);
  const int KP = 18 * ((p.C_in + 1) / 2);
  unsigned* wa = (unsigned*)workspace;
  unsigned* wb = (unsigned*)((char*)workspace + align256(n_pairs * 4));
  const unsigned blocks = (unsigned)min((n_pairs + 255) / 256, (size_t)4096);
  const unsigned* wp_min = nullptr;
  const unsigned* wp_max = nullptr;
  if (p.mode == TCONV_PARALLEL) {
    hipLaunchKernelGGL(relay_pairs_kernel, dim3(blocks), dim3(256), 0, s, (const unsigned short*)a.w_min, wa, p.C_out, p.K, KP);
    hipLaunchKernelGGL(relay_pairs_kernel, dim3(blocks), dim3(256), 0, s, (const unsigned short*)a.w_max, wb, p.C_out, p.K, KP);
    wp_min = wa; wp_max = wb;
  } else {
    const void* w = (p.mode == TCONV_MIN) ? a.w_min : a.w_max;
    hipLaunchKernelGGL(relay_pairs_kernel, dim3(blocks), dim3(256), 0, s, (const unsigned short*)w, wa, p.C_out, p.K, KP);
    wp_min = wp_max = wa;
  }
  switch (p.mode) {
    case TCONV_MAX: return launch_m<TCONV_MAX>(p, a, wp_min, wp_max, s);
    case TCONV_MIN: return launch_m<TCONV_MIN>(p, a, wp_min, wp_max, s);
    case TCONV_COMPOUND: return launch_m<TCONV_COMPOUND>(p, a, wp_min, wp_max, s);
    default: return launch_m<TCONV_PARALLEL>(p, a, wp_min, wp_max, s);
  }
}

}  // namespace tconv
