// The tiled 3x3 forward kernel and its launcher, as templates: each of the translation units that instantiate them
// (the plain form, the form with the input region staged in LDS, the form that splits the input channels over the
// waves of a workgroup) is a code object of its own, so that none grows past what the loader has been seen to take.
//
// Tiled forward kernel for 3x3 tropical convolutions on gfx950: a VALU "semiring GEMM".
//
// Operator: paper Sec. 3.1 layers (iv) / (v) (one min / max over all C_in*9 taps of x + w) and the
// Sec. 3.3 compound (one shared add feeds both reductions, Sec. 3.5 closing remark) and parallel
// combinations, and the Sec. 3.1 mixed layers (iii) / (vi) (min-plus inside a channel under a max over
// the channels, and the dual), which differ only in the inner block.  The semiring has no multiply, so the matrix cores do not apply; the kernel is
// built for the vector ALUs:
//
//  * A lane owns a row segment of PX consecutive output pixels (8 at stride 1, 4 at stride 2) and 4
//    output channels: 4*PX running extrema per branch stay in VGPRs for the whole K loop.  The 4
//    waves of a workgroup share the pixel segments (same x lines in L1) and differ in output-channel
//    group.  The main loop uses no LDS and no barrier.
//  * Kernel values are wave-uniform: scalar loads straight from the OIHW tensor (k is contiguous
//    per c_out) put the 18 values of a channel pair in SGPRs, where they are the scalar operand
//    of v_add_f32 - no repacking pass, no VGPRs, no LDS.
//  * Implicit im2col: per channel a lane loads 3 rows x ((PX-1)*stride + 2*dil + 1) input values
//    once (raw buffer loads: wave-uniform descriptor + 32-bit lane offset + uniform channel offset)
//    and reuses them for 9 taps x PX pixels x 4 channels.  Padding becomes NaN with one OR per loaded
//    value; v_max/v_min/v_max3/v_min3 return the non-NaN operand, so a padded tap never wins in
//    either branch and costs nothing in the inner loop.
//  * Inner blocks (tile_blocks_gfx950.h, hand-scheduled): one accumulator walks two channels
//    (18 taps) with 18 adds, v_max3/v_min3 chains, and 2 compares + 2 selects per branch that
//    record the winning CHANNEL.  After the K loop the epilogue re-evaluates the 9 taps of that
//    channel and takes the first that equals the extremum: exactly the lowest winning tap.
//  * Register-resident software pipeline for the six x rows of a channel pair.  Stride 1: six slots;
//    pixels are walked left to right, so the low columns of every slot die first and are re-loaded
//    for the NEXT channel pair in the middle of the current one, the high columns at its end.
//    Stride 2: the rows are short, two full sets of slots alternate (the pair loop is unrolled by two).
//    Masks are applied just before the first use.
#pragma once
#include <stdlib.h>

#include "tile_common.h"
// after tile_common.h: the blocks header relies on the HIP runtime declarations included there
#include <tile_blocks_gfx950.h>


namespace tconv {
namespace {

using namespace tile;

// the epilogue's operands as a kernel argument (device pointers, NULL = step left out)
struct Epilogue {
  const float* bias;
  const float* scale;
  const float* shift;
  const void* residual;
};

// kernel flag: keep the hardware's workgroup order (tuning builds only)
constexpr int FLAG_ROUND_ROBIN = 32;

// 9 x values of pixel q for the 3x3 taps of one channel: rows[3*ch + i][q*S + j*D]
template <int S, int D, int XR>
__device__ __forceinline__ void taps_of(float (&out)[9], const float (&rows)[6][XR], int ch, int q) {
#pragma unroll
  for (int i = 0; i < 3; ++i)
#pragma unroll
    for (int j = 0; j < 3; ++j) out[i * 3 + j] = rows[ch * 3 + i][q * S + j * D];
}

// TN: output channels per lane (4; 2 for layers too small to fill the chip with 4)
// PZ: zero padding (App. A.1.1: the unfold formulation pads with zeros): an out-of-image value is +0 instead of NaN,
//     so its tap competes like any other; one AND per loaded value where the identity padding has one OR
// XA: bf16 storage at stride 1: every lane's core columns start at an even element of x, so they are read as
//     whole dwords holding two values each (otherwise bf16 values are read one by one); fp32 storage at stride 2: the
//     right halo column is inside the row for every lane and is read in one run with the core columns
// KSP: the four waves of a workgroup share ONE group of TN output channels and split the input channels between
//     them (a quarter of the channel pairs each, in ascending order); their running extrema and winning channels
//     meet in LDS, wave w keeps output channel w of the group and finishes it.  Four times as many, a quarter as
//     long workgroups: for layers whose grid is a few workgroups per compute unit at most, where whole rounds of
//     equally long workgroups leave the chip part empty at the end, or never fill it.
template <int MODE, int S, int D, int TN, bool PZ, typename TO, bool XA, bool KSP>
__global__ __launch_bounds__(WAVES * 64, 2) void fwd_tiled3x3_kernel(
    Params p, const TO* __restrict__ x, const float* __restrict__ w_min,
    const float* __restrict__ w_max, const float* __restrict__ alpha,
    const float* __restrict__ beta, TO* __restrict__ y, TO* __restrict__ y_min,
    TO* __restrict__ y_max, int32_t* __restrict__ idx_min, int32_t* __restrict__ idx_max, Epilogue ep, int segs,
    int n_units, int n_groups, int wrps, int flags, int n_ublocks, int xsplit) {
  // the mixed layers run as one branch: (iii) through the min-side kernel, accumulators and outputs
  // (its operator is min-plus), (vi) through the max side; only the start value and the block differ
  constexpr bool DO_MIN = mode_has_min(MODE), DO_MAX = mode_has_max(MODE);
  constexpr int PX = (S == 1) ? 8 : 4;          // output pixels per lane
  constexpr int NC = (PX - 1) * S + 1;          // core columns [D, D+NC): always inside the row
  constexpr int XR = NC + 2 * D;                // input columns a lane touches per row
  constexpr bool PK = XA && sizeof(TO) == 2 && S == 1;  // core columns arrive two per dword
  // stride 2, fp32 storage, XA: the right halo column lies inside the row for every lane (the host has checked), so
  // the 7 core columns and it are one run of 8 values (two 16-byte loads instead of a 16-, an 8-, a 4-byte load and a
  // single value: at stride 2 the texture addresser is the busiest unit)
  constexpr bool WIDE2 = XA && sizeof(TO) == 4 && S == 2;
  // the same at stride 2 in 16-bit storage, where the run also starts at an even element: four dwords of two values
  constexpr bool PK2 = XA && sizeof(TO) == 2 && S == 2;

  // ---- which c_out group (wave-uniform) and which pixel segment (per lane)
  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2: XCD = blockIdx & 7.  A workgroup is a
  // (pixel block, output-channel block) pair; the workgroups of one pixel block read the same input lines, those of
  // one channel block the same kernel rows.  The XCDs split the work two ways: xsplit (1, 2, 4 or 8) parts of the
  // channel blocks times 8 / xsplit parts of the pixel blocks, so that an XCD's share of the kernel tensors stays
  // within reach of its L2 while every input line is fetched by xsplit XCDs instead of all eight.  Inside an XCD the
  // channel blocks of a pixel block are numbered consecutively.
  const int gblocks = KSP ? n_groups : (n_groups + WAVES - 1) / WAVES;
  int ublock, gblock;
  if (flags & FLAG_ROUND_ROBIN) {
    if ((int)blockIdx.x >= n_ublocks * gblocks) return;
    ublock = (int)blockIdx.x / gblocks;
    gblock = (int)blockIdx.x - ublock * gblocks;
  } else {
    const int xcd = (int)(blockIdx.x & 7u), j = (int)(blockIdx.x >> 3);
    const int gb_per = (gblocks + xsplit - 1) / xsplit;
    const int pparts = 8 / xsplit;
    const int ub_per = (n_ublocks + pparts - 1) / pparts;
    const int lu = j / gb_per, lg = j - lu * gb_per;
    ublock = (xcd / xsplit) * ub_per + lu;
    gblock = (xcd & (xsplit - 1)) * gb_per + lg;
    // padding of the grid (whole workgroups leave; the kernel has no barrier)
    if (lu >= ub_per || ublock >= n_ublocks || gblock >= gblocks) return;
  }
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int group = KSP ? gblock : gblock * WAVES + wave;
  const size_t HW = (size_t)p.H * p.W;
  // x is read in its storage type TO: fp32, or bf16 whose 16 bits are the upper half of the fp32 value (the widening
  // shift is fused with the padding mask, see mask_cols)
  const rsrc_t xres = make_rsrc(x, (unsigned)((size_t)p.N * p.C_in * HW * sizeof(TO)));
  HIP_DYNAMIC_SHARED(float, dyn_lds)
  const int KS = (p.K + 3) & ~3;  // stride of a kernel row staged in LDS (epilogue)
  if (!KSP && group >= n_groups) return;  // whole wave leaves; no barrier follows
  const int co0 = group * TN;
  const int lane = threadIdx.x & 63;
  const int unit_raw = ublock * 64 + lane;
  const bool unit_ok = unit_raw < n_units;
  const int unit = unit_ok ? unit_raw : n_units - 1;  // surplus lanes recompute the last unit, store nothing
  const int seg = unit % segs;
  const int oh = (unit / segs) % p.Ho;
  const int n = unit / (segs * p.Ho);
  // the last segment of a row is shifted left so that every lane owns PX real pixels;
  // pixels it shares with its neighbour are computed twice and stored once
  const int ow_nom = seg * PX;
  const int ow0 = min(ow_nom, p.Wo - PX);
  const int first_q = ow_nom - ow0;

  // ---- channel-independent addressing and padding masks
  const int iw0 = ow0 * S - p.pw;  // input column of register column 0
  unsigned roff[3];  // byte offset of the first core column (iw0 + D >= 0) of each (clamped) row
  unsigned mrow[3];  // identity padding: all-ones where the row is padding; zero padding: all-ones where it is NOT
  int ihc[3];        // clamped input rows of the three kernel rows
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int ih = oh * S - p.ph + i * D;
    mrow[i] = ((ih >= 0 && ih < p.H) != PZ) ? 0u : 0xffffffffu;
    ihc[i] = min(max(ih, 0), p.H - 1);
    roff[i] = (unsigned)(((size_t)n * p.C_in * HW + (size_t)ihc[i] * p.W + (size_t)(iw0 + D)) * sizeof(TO));
  }
  int hoff[2 * D];         // clamped byte offsets of the halo columns relative to roff
  unsigned mhalo[2 * D];   // the same two conventions for the halo columns
#pragma unroll
  for (int h = 0; h < 2 * D; ++h) {
    const int o = (h < D) ? h : h + NC;
    const int iw = iw0 + o;
    mhalo[h] = ((iw >= 0 && iw < p.W) != PZ) ? 0u : 0xffffffffu;
    hoff[h] = (min(max(iw, 0), p.W - 1) - (iw0 + D)) * (int)sizeof(TO);
  }

  // ---- kernel rows of this wave's output channels (wave-uniform)
  const float* wr_min[TN];
  const float* wr_max[TN];
#pragma unroll
  for (int c = 0; c < TN; ++c) {
    const int co = min(co0 + c, p.C_out - 1);
    wr_min[c] = DO_MIN ? w_min + (size_t)co * p.K : nullptr;
    wr_max[c] = DO_MAX ? w_max + (size_t)co * p.K : nullptr;
  }

  float bmax[TN][PX], bmin[TN][PX];
  int imax[TN][PX], imin[TN][PX];
#pragma unroll
  for (int c = 0; c < TN; ++c)
#pragma unroll
    for (int q = 0; q < PX; ++q) {
      bmax[c][q] = (MODE == TCONV_MAXPLUS_MIN) ? INFINITY : -INFINITY;   // identity of the fold over channels
      bmin[c][q] = (MODE == TCONV_MINPLUS_MAX) ? -INFINITY : INFINITY;
      imax[c][q] = 0; imin[c][q] = 0;
    }

  // ---- main loop over channel pairs (cA = 2*du, cB = 2*du + 1; an odd C_in gets a virtual last
  // channel whose x is all NaN)
#ifdef TCONV_TUNING
  const int ndu_all = (flags & 2) ? 0 : (p.C_in + 1) >> 1;  // timing experiment: no main loop, WRONG results
#else
  const int ndu_all = (p.C_in + 1) >> 1;
#endif
  // the pairs [du_lo, ndu) this wave walks: all of them, or its quarter
  const int du_per = (ndu_all + WAVES - 1) / WAVES;
  const int du_lo = KSP ? min(wave * du_per, ndu_all) : 0;
  const int ndu = KSP ? min(du_lo + du_per, ndu_all) : ndu_all;

  auto chan_soff = [&](int c) -> unsigned {  // wave-uniform byte offset of channel c (clamped)
    return (unsigned)((size_t)min(c, p.C_in - 1) * HW * sizeof(TO));
  };
  // loads of columns [lo, hi) of all six rows of channel pair du; lo / hi fall on the boundaries
  // {0, D, D+4, D+NC, XR} so that every piece is a halo single or a run of the core
  auto issue_cols = [&](float (&xs)[6][XR], int du, int lo, int hi) {
#pragma unroll
    for (int sl = 0; sl < 6; ++sl) {
      const unsigned soff = chan_soff(2 * du + sl / 3);
      const unsigned ro = roff[sl % 3];
      if (lo == 0) {
#pragma unroll
        for (int h = 0; h < D; ++h) xs[sl][h] = load_raw_one<TO>(xres, ro + (unsigned)hoff[h], soff);
      }
      if constexpr (PK) {
        // dwords of two values: columns D .. D+3 land in slots D, D+1 and columns D+4 .. D+7 in slots D+4, D+5;
        // mask_cols spreads them over the slots of their columns
        if (lo <= D) load_run<2, float>(&xs[sl][D], xres, ro, soff);
        if (hi >= D + NC) load_run<2, float>(&xs[sl][D + 4], xres, ro + 8u, soff);
      } else if constexpr (PK2) {
        load_run<4, float>(&xs[sl][D], xres, ro, soff);  // 8 values in slots D .. D+3; mask_cols spreads them
      } else if constexpr (WIDE2) {
        load_raw_run<NC + D, TO>(&xs[sl][D], xres, ro, soff);  // always called for whole rows at stride 2
      } else if (lo <= D && hi >= D + NC) {
        load_raw_run<NC, TO>(&xs[sl][D], xres, ro, soff);
      } else if (lo <= D) {
        load_raw_run<4, TO>(&xs[sl][D], xres, ro, soff);                                      // first 4 core columns
      } else {
        load_raw_run<NC - 4, TO>(&xs[sl][D + 4], xres, ro + 4u * (unsigned)sizeof(TO), soff);  // the rest of the core
      }
      if (hi == XR && !WIDE2 && !PK2) {
#pragma unroll
        for (int h = 0; h < D; ++h) xs[sl][D + NC + h] = load_raw_one<TO>(xres, ro + (unsigned)hoff[D + h], soff);
      }
    }
  };
  // padding -> NaN (identity) or +0 (zero padding), columns [lo, hi); the virtual channel of an odd C_in -> NaN always.
  // bf16 storage: a slot holds the 16 loaded bits until here; the widening shift and the mask are ONE instruction
  // ((v << 16) | m), so that bf16 rows cost the main loop no more than fp32 rows and half the bytes.
  auto mask_cols = [&](float (&xs)[6][XR], int lo, int hi, unsigned mB) {
#pragma unroll
    for (int sl = 0; sl < 6; ++sl) {
      const unsigned vB = sl >= 3 ? mB : 0u;
      const unsigned mr = PZ ? mrow[sl % 3] : (mrow[sl % 3] | vB);
      if constexpr (PK) {
        // both dwords of a half are read before any slot of the half is written
        unsigned pk[4];
#pragma unroll
        for (int h = 0; h < 4; ++h) pk[h] = __float_as_uint(xs[sl][D + (h & 1) + (h >> 1) * 4]);
#pragma unroll
        for (int h = 0; h < 4; ++h) {
          if (D + 2 * h < lo || D + 2 * h >= hi) continue;
          const unsigned v0 = pk[h] << 16, v1 = pk[h] & 0xffff0000u;
          xs[sl][D + 2 * h] = __uint_as_float(PZ ? ((v0 & mr) | vB) : (v0 | mr));
          xs[sl][D + 2 * h + 1] = __uint_as_float(PZ ? ((v1 & mr) | vB) : (v1 | mr));
        }
      }
      if constexpr (PK2) {
        // columns D .. D+7 (the core and the right halo column) from the four dwords, all read before any is written
        unsigned pk[4];
#pragma unroll
        for (int h = 0; h < 4; ++h) pk[h] = __float_as_uint(xs[sl][D + h]);
#pragma unroll
        for (int h = 0; h < 4; ++h) {
          const unsigned v0 = pk[h] << 16, v1 = pk[h] & 0xffff0000u;
          const int o1 = D + 2 * h + 1;
          unsigned m1 = mr;
          if (o1 >= D + NC) m1 = PZ ? (m1 & mhalo[o1 - NC]) : (m1 | mhalo[o1 - NC]);
          xs[sl][D + 2 * h] = __uint_as_float(PZ ? ((v0 & mr) | vB) : (v0 | mr));
          xs[sl][o1] = __uint_as_float(PZ ? ((v1 & m1) | vB) : (v1 | m1));
        }
      }
#pragma unroll
      for (int o = 0; o < XR; ++o) {
        if (o < lo || o >= hi) continue;
        if (PK && o >= D && o < D + NC) continue;
        if (PK2 && o >= D) continue;
        unsigned m = mr;
        if (o < D) m = PZ ? (m & mhalo[o]) : (m | mhalo[o]);
        if (o >= D + NC) m = PZ ? (m & mhalo[o - NC]) : (m | mhalo[o - NC]);
        const unsigned raw = __float_as_uint(xs[sl][o]);
        const unsigned val = sizeof(TO) == 2 ? raw << 16 : raw;
        xs[sl][o] = __uint_as_float(PZ ? ((val & m) | vB) : (val | m));
      }
    }
  };
  // 18 kernel values (channels cA, cB) of output channel slot c; the offsets are laundered so that
  // every block re-loads them (SGPRs are too few to keep all four channels' values live)
  auto load_w = [&](float (&wv)[18], const float* row, int cA, int cB) {
    const float* pa = row + launder_uniform(cA * 9);
    const float* pb = row + launder_uniform(cB * 9);
#pragma unroll
    for (int t = 0; t < 9; ++t) { wv[t] = pa[t]; wv[9 + t] = pb[t]; }
  };
  // the blocks of pixels [q_lo, q_hi) for all four channels; wc carries the kernel values of the
  // next block to run (they are fetched one block ahead)
  constexpr int QSTEP = (MODE == TCONV_COMPOUND) ? 1 : 2;  // single-branch blocks cover two pixels
  auto do_pixels = [&](float (&xs)[6][XR], float (&wc)[18], int q_lo, int q_hi, int cA, int cB, int tA, int tB) {
#pragma unroll
    for (int q = q_lo; q < q_hi; q += QSTEP) {
      if (MODE == TCONV_COMPOUND) {
        float xA[9], xB[9];
        taps_of<S, D, XR>(xA, xs, 0, q);
        taps_of<S, D, XR>(xB, xs, 1, q);
#pragma unroll
        for (int c = 0; c < TN; ++c) {
          float wn[18];
          load_w(wn, wr_max[(c + 1) % TN], cA, cB);
          float wA[9], wB[9];
#pragma unroll
          for (int t = 0; t < 9; ++t) { wA[t] = wc[t]; wB[t] = wc[9 + t]; }
          blk_both(bmax[c][q], bmin[c][q], imax[c][q], imin[c][q], xA, xB, wA, wB, tA, tB);
#pragma unroll
          for (int t = 0; t < 18; ++t) wc[t] = wn[t];
        }
      } else {
        // parallel mode runs a max block and a min block per pixel pair
        constexpr int NB = (MODE == TCONV_PARALLEL) ? 2 : 1;
        float xA0[9], xB0[9], xA1[9], xB1[9];
        taps_of<S, D, XR>(xA0, xs, 0, q);
        taps_of<S, D, XR>(xB0, xs, 1, q);
        taps_of<S, D, XR>(xA1, xs, 0, q + 1);
        taps_of<S, D, XR>(xB1, xs, 1, q + 1);
#pragma unroll
        for (int c = 0; c < TN; ++c)
#pragma unroll
          for (int b = 0; b < NB; ++b) {
            const bool is_max = (MODE == TCONV_MAX) || (MODE == TCONV_MAXPLUS_MIN) || (MODE == TCONV_PARALLEL && b == 0);
            // next block in program order: other branch of the same channel, or next channel
            const int cn = (b == NB - 1) ? (c + 1) % TN : c;
            const bool next_is_max = (MODE == TCONV_MAX) || (MODE == TCONV_MAXPLUS_MIN) ||
                                     (MODE == TCONV_PARALLEL && ((b + 1) % NB) == 0);
            float wn[18];
            load_w(wn, next_is_max ? wr_max[cn] : wr_min[cn], cA, cB);
            float wA[9], wB[9];
#pragma unroll
            for (int t = 0; t < 9; ++t) { wA[t] = wc[t]; wB[t] = wc[9 + t]; }
            if (MODE == TCONV_MAXPLUS_MIN)
              blk_maxmin2(bmax[c][q], imax[c][q], bmax[c][q + 1], imax[c][q + 1], xA0, xB0, xA1, xB1, wA, wB, tA, tB);
            else if (MODE == TCONV_MINPLUS_MAX)
              blk_minmax2(bmin[c][q], imin[c][q], bmin[c][q + 1], imin[c][q + 1], xA0, xB0, xA1, xB1, wA, wB, tA, tB);
            else if (is_max)
              blk_max2(bmax[c][q], imax[c][q], bmax[c][q + 1], imax[c][q + 1], xA0, xB0, xA1, xB1, wA, wB, tA, tB);
            else
              blk_min2(bmin[c][q], imin[c][q], bmin[c][q + 1], imin[c][q + 1], xA0, xB0, xA1, xB1, wA, wB, tA, tB);
#pragma unroll
            for (int t = 0; t < 18; ++t) wc[t] = wn[t];
          }
      }
    }
  };
  const float* w_first = DO_MAX ? wr_max[0] : wr_min[0];  // kernel row of the first block of a pair

  if constexpr (S == 1) {
    // six slots, column-phased: columns [0, H1) are dead once pixel P1 is done and are first needed
    // again at pixel 0; columns [H1, XR) are first read by pixel P2
    constexpr int H1 = D + 4;
    constexpr int QA = (4 - D) & ~(QSTEP - 1);            // first pixel (block start) reading column H1
    constexpr int QB = ((D + 3) | (QSTEP - 1)) + 1;       // first pixel after the last reader of column H1 - 1
    float xs[6][XR];
    if (ndu > du_lo) issue_cols(xs, du_lo, 0, XR);
    for (int du = du_lo; du < ndu; ++du) {
      const int dn = min(du + 1, ndu - 1);  // past the end: re-load the last pair (unused, in bounds)
      const int cA = 2 * du, cBv = 2 * du + 1, cB = min(cBv, p.C_in - 1);
      const unsigned mB = (cBv < p.C_in) ? 0u : 0xffffffffu;
      float wc[18];
      load_w(wc, w_first, cA, cB);
      mask_cols(xs, 0, H1, mB);
      do_pixels(xs, wc, 0, QA, cA, cB, cA, cBv);
      mask_cols(xs, H1, XR, mB);
      do_pixels(xs, wc, QA, QB, cA, cB, cA, cBv);
      issue_cols(xs, dn, 0, H1);
      do_pixels(xs, wc, QB, PX, cA, cB, cA, cBv);
      issue_cols(xs, dn, H1, XR);
    }
  } else {
    // two sets of six slots: the rows of the next pair are loaded while the current pair runs
    float xs0[6][XR], xs1[6][XR];
    if (ndu > du_lo) issue_cols(xs0, du_lo, 0, XR);
    for (int du = du_lo; du < ndu; du += 2) {
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int d = du + half;
        if (d < ndu) {  // wave-uniform
          const int dn = min(d + 1, ndu - 1);
          const int cA = 2 * d, cBv = 2 * d + 1, cB = min(cBv, p.C_in - 1);
          const unsigned mB = (cBv < p.C_in) ? 0u : 0xffffffffu;
          float wc[18];
          load_w(wc, w_first, cA, cB);
          if (half == 0) {
            issue_cols(xs1, dn, 0, XR);
            mask_cols(xs0, 0, XR, mB);
            do_pixels(xs0, wc, 0, PX, cA, cB, cA, cBv);
          } else {
            issue_cols(xs0, dn, 0, XR);
            mask_cols(xs1, 0, XR, mB);
            do_pixels(xs1, wc, 0, PX, cA, cB, cA, cBv);
          }
        }
      }
    }
  }

  // ---- epilogue: exact tap of every extremum (first tap of the winning channel, in k order, whose
  // sum equals it), combine, store.  Each lane writes its PX consecutive outputs with 16-byte stores.
  // The winning-channel ids are parked in LDS (16 bits each, a private slot per lane: no barrier)
  // so that the gather batches below have registers to land in.
  constexpr int NBR = (DO_MIN && DO_MAX) ? 2 : 1;
  constexpr int NST = KSP ? 1 : NBR;  // KSP: one branch at a time goes through the exchange below
  __shared__ int stash[WAVES][NST][TN][PX / 2][64];
  float fmin[PX], fmax[PX];  // KSP: extrema and winning channels of the output channel this wave finishes
  int jmin[PX], jmax[PX];
  if constexpr (KSP) {
    // Every wave hands its extrema and winning channels of one branch to LDS; wave w folds the four candidates of
    // output channel w in wave order = ascending input channels, replacing only on a strict improvement: the lowest
    // channel that reaches the extremum, as in the undivided scan.
    __shared__ float xch[WAVES][TN][PX][64];
    auto exchange = [&](const float (&b)[TN][PX], const int (&id)[TN][PX], bool larger_wins, float (&fb)[PX],
                        int (&fj)[PX]) {
#pragma unroll
      for (int c = 0; c < TN; ++c) {
#pragma unroll
        for (int q = 0; q < PX; ++q) xch[wave][c][q][lane] = b[c][q];
#pragma unroll
        for (int h = 0; h < PX / 2; ++h) stash[wave][0][c][h][lane] = id[c][2 * h] | (id[c][2 * h + 1] << 16);
      }
      __syncthreads();
      const int cw = min(wave, TN - 1);
#pragma unroll
      for (int q = 0; q < PX; ++q) {
        float best = xch[0][cw][q][lane];
        unsigned pk = (unsigned)stash[0][0][cw][q >> 1][lane];
        int bid = (q & 1) ? (int)(pk >> 16) : (int)(pk & 0xffffu);
#pragma unroll
        for (int w2 = 1; w2 < WAVES; ++w2) {
          const float v = xch[w2][cw][q][lane];
          pk = (unsigned)stash[w2][0][cw][q >> 1][lane];
          const int vid = (q & 1) ? (int)(pk >> 16) : (int)(pk & 0xffffu);
          const bool better = larger_wins ? (v > best) : (v < best);
          best = better ? v : best;
          bid = better ? vid : bid;
        }
        fb[q] = best; fj[q] = bid;
      }
      __syncthreads();  // the buffers are free for the next branch
    };
    if (DO_MIN) exchange(bmin, imin, MODE == TCONV_MINPLUS_MAX, fmin, jmin);
    if (DO_MAX) exchange(bmax, imax, MODE != TCONV_MAXPLUS_MIN, fmax, jmax);
    if (wave >= TN || co0 + wave >= p.C_out) return;  // no barrier follows
  } else {
#pragma unroll
    for (int c = 0; c < TN; ++c)
#pragma unroll
      for (int h = 0; h < PX / 2; ++h) {
        if (DO_MIN) stash[wave][0][c][h][lane] = imin[c][2 * h] | (imin[c][2 * h + 1] << 16);
        if (DO_MAX) stash[wave][NBR - 1][c][h][lane] = imax[c][2 * h] | (imax[c][2 * h + 1] << 16);
      }
  }
  auto unstash = [&](int br, int c, int (&ids)[PX]) {
#pragma unroll
    for (int h = 0; h < PX / 2; ++h) {
      const unsigned a2 = (unsigned)stash[wave][KSP ? 0 : br][c][h][lane];
      ids[2 * h] = (int)(a2 & 0xffffu); ids[2 * h + 1] = (int)(a2 >> 16);
    }
  };
  const int first_qs = unit_ok ? first_q : PX;  // surplus lanes store nothing (they still help with the copies below)
  const size_t wbytes = (size_t)p.C_out * p.K * sizeof(float);
  const rsrc_t wres_min = make_rsrc(DO_MIN ? w_min : w_max, (unsigned)wbytes);
  const rsrc_t wres_max = make_rsrc(DO_MAX ? w_max : w_min, (unsigned)wbytes);
  const size_t xn_off = (size_t)n * p.C_in * HW;
  // The kernel values the gathers need are one K-float row per (output channel, branch); a gather
  // straight from global memory costs the texture addresser one address per lane, so the wave first
  // copies wrps such rows (as many as fit its share of LDS; 0: none fit) with coalesced loads and
  // gathers from LDS.  Rows are numbered in the order they are used: c * NT + t.
  constexpr int NT = (MODE == TCONV_PARALLEL) ? 2 : 1;  // kernel tensors
  float* const wstage = dyn_lds + wave * (wrps * KS);
  auto stage_rows = [&](int s0) {
    wave_lds_fence();  // every lane is done with the rows staged before
    for (int r = 0; r < wrps; ++r) {
      const int s = s0 + r;
      if (s >= (KSP ? 1 : TN) * NT) break;
      const int co = min(co0 + (KSP ? wave : 0) + s / NT, p.C_out - 1);
      const bool use_max = DO_MAX && (NT == 1 || (s % NT) == 1);
      const unsigned rbase = (unsigned)((size_t)co * p.K * sizeof(float));
      float* const dst = wstage + r * KS;
      // 4 floats per lane and trip; the last chunk of the row is moved back so that it ends with the row
      for (int f = lane * 4; f < p.K; f += 256) {
        const int fs = min(f, p.K - 4);
        float v[4];
        load_run<4, float>(v, use_max ? wres_max : wres_min, rbase + (unsigned)fs * 4u, 0u);
#pragma unroll
        for (int t = 0; t < 4; ++t) dst[fs + t] = v[t];
      }
    }
    wave_lds_fence();
  };
  // Exact taps for RB pixels of one (channel, branch) row at a time: first ALL gathers of the batch
  // are issued (9 kernel values and a 3 x (2D+1) input patch per item), only then any is consumed,
  // so the batch pays one memory latency instead of one per item.  Straight-line code: the pixel index is a
  // compile-time constant, an out-of-image tap is masked exactly as in the main loop (NaN, or +0 under zero
  // padding) and so needs no test of its own, and what depends on the lane alone (row offsets, the start column
  // of every pixel's patch, its shift) is computed once for all items.
  constexpr int L = 2 * D + 1;           // contiguous input columns spanned by the 3 taps of a row
  constexpr int RB = (D == 1) ? 4 : 2;   // items per batch (register budget)
  constexpr int ND16 = (L + 2) / 2;      // 16-bit storage: aligned dwords that cover L values from any halfword
  // a pixel whose three tap columns are core columns (always inside the row) loads its patch where it is; the
  // others load from a start clamped into the row and pick their taps by the shift
  auto is_inner = [](int q) { return q * S >= D && q * S + 2 * D < D + NC; };
  const unsigned HWb = (unsigned)(HW * sizeof(TO));
  unsigned rowb[3];   // byte offset of column 0 of the (clamped) input row i in channel 0 of this image
  unsigned colb[PX];  // byte offset of the first loaded column of pixel q's patch
  int shq[PX];        // non-inner pixels: tap column minus loaded column
#pragma unroll
  for (int i = 0; i < 3; ++i) rowb[i] = (unsigned)((xn_off + (size_t)ihc[i] * p.W) * sizeof(TO));
#pragma unroll
  for (int q = 0; q < PX; ++q) {
    const int iwq = iw0 + q * S;
    const int start = is_inner(q) ? iwq : min(max(iwq, 0), p.W - L);
    colb[q] = (unsigned)start * (unsigned)sizeof(TO);
    shq[q] = iwq - start;
  }
  // the padding mask of the tap in register column o of row i, in the convention of the main loop
  auto tap_mask = [&](int i, int o) -> unsigned {
    unsigned m = mrow[i];
    if (o < D) m = PZ ? (m & mhalo[o]) : (m | mhalo[o]);
    if (o >= D + NC) m = PZ ? (m & mhalo[o - NC]) : (m | mhalo[o - NC]);
    return m;
  };
  auto refine_batch = [&](auto q0c, const int (&cs_row)[PX], const float (&best_row)[PX], rsrc_t wres, int co,
                          const float* wl, int (&res)[PX]) {
    constexpr int q0 = decltype(q0c)::value;
    float wv[RB][9];
    float run[RB][3][L];
    int csv[RB];
    static_steps<0, RB, 1>([&](auto uc) {
      constexpr int u = decltype(uc)::value, q = q0 + u;
      const int cs = min(cs_row[q], p.C_in - 1);  // a virtual channel never wins; keep the address in range
      csv[u] = cs;
      if (wl) {  // uniform
#pragma unroll
        for (int t = 0; t < 9; ++t) wv[u][t] = wl[cs * 9 + t];
      } else {
        load_run<9, float>(wv[u], wres, (unsigned)(((size_t)co * p.K + (size_t)cs * 9) * sizeof(float)), 0u);
      }
      const unsigned xb = (unsigned)cs * HWb + colb[q];
#pragma unroll
      for (int i = 0; i < 3; ++i) {
        if constexpr (sizeof(TO) == 2) {
          // 16-bit storage: the aligned dwords that cover the L values (one load; unpacked below, after the batch's
          // loads are all out).  The host takes this kernel only for a dword-aligned x with an even element count,
          // so the last dword of a run never reaches past the tensor.
          load_run<ND16, float>(run[u][i], xres, (xb + rowb[i]) & ~3u, 0u);
        } else {
          load_run<L, TO>(run[u][i], xres, xb + rowb[i], 0u);
        }
      }
    });
    __builtin_amdgcn_sched_barrier(0);  // keep the gathers of the batch ahead of every use
    static_steps<0, RB, 1>([&](auto uc) {
      constexpr int u = decltype(uc)::value, q = q0 + u;
      constexpr bool inner = q * S >= D && q * S + 2 * D < D + NC;
      int rt = 0;  // winning tap inside the channel
      if constexpr (sizeof(TO) == 2) {
        // shift the dword run right by the halfword the values start at, then widen value t from half t of the run
        const unsigned xb = (unsigned)csv[u] * HWb + colb[q];
#pragma unroll
        for (int i = 0; i < 3; ++i) {
          const unsigned sh = ((xb + rowb[i]) & 2u) << 3;
          unsigned r[ND16];
#pragma unroll
          for (int k = 0; k < ND16; ++k) {
            const unsigned lo = __float_as_uint(run[u][i][k]);
            r[k] = k + 1 < ND16 ? __builtin_amdgcn_alignbit(__float_as_uint(run[u][i][k + 1]), lo, sh) : lo >> sh;
          }
#pragma unroll
          for (int t = 0; t < L; ++t)
            run[u][i][t] = __uint_as_float((t & 1) ? (r[t >> 1] & 0xffff0000u) : (r[t >> 1] << 16));
        }
      }
#pragma unroll
      for (int i = 2; i >= 0; --i) {
        // identity padding, inner pixel: only a whole row can be outside; its taps are compared with NaN
        const float best_i = (!PZ && inner) ? nan_or(best_row[q], mrow[i]) : best_row[q];
#pragma unroll
        for (int j = 2; j >= 0; --j) {
          float xv;
          if constexpr (inner) {
            xv = run[u][i][j * D];
          } else {
            const int col = j * D + shq[q];  // position of the tap inside the loaded run
            xv = run[u][i][0];
#pragma unroll
            for (int t = 1; t < L; ++t) xv = (col == t) ? run[u][i][t] : xv;
          }
          // an out-of-image tap: no candidate (identity padding: NaN), or the candidate 0 + w (zero padding)
          if constexpr (PZ || !inner) {
            const unsigned m = tap_mask(i, q * S + j * D);
            xv = __uint_as_float(PZ ? (__float_as_uint(xv) & m) : (__float_as_uint(xv) | m));
          }
          const float sum = __fadd_rn(xv, wv[u][i * 3 + j]);
          rt = (sum == best_i) ? i * 3 + j : rt;
        }
      }
#ifdef TCONV_TUNING
      res[q] = (flags & 1) ? csv[u] * 9 : csv[u] * 9 + rt;  // timing experiment: no tap recovery, WRONG results
#else
      res[q] = csv[u] * 9 + rt;
#endif
    });
    __builtin_amdgcn_sched_barrier(0);  // the next batch starts after this one has retired its registers
  };
  const size_t plane = (size_t)p.Ho * p.Wo;
  const unsigned lane_ob = (unsigned)(((size_t)n * p.C_out) * plane + (size_t)oh * p.Wo + ow0);
  // one output channel: c is its slot among the parked winners and the staged kernel rows
  auto finish_channel = [&](int c, int co, const float (&vmin)[PX], const float (&vmax)[PX]) {
    // outputs: a wave-uniform channel base and the lane's 32-bit element offset (tensors stay below 4 GiB)
    const size_t cb_off = (size_t)co * plane;
    const size_t ob = lane_ob + cb_off;
    float ca = 1.f, cb = 1.f;
    if (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL) {
      if (alpha) ca = alpha[co];
      if (beta) cb = beta[co];
    }
    int ridx[PX], cids[PX];
    float out[PX];
    // rows of this channel in use order: parallel: min row, then max row; else the one row
    const int s_min = c * NT, s_max = c * NT + (NT - 1);
    if (DO_MIN) {
      if (wrps > 0 && s_min % wrps == 0) stage_rows(s_min);
      const float* wl = wrps > 0 ? wstage + (s_min % wrps) * KS : nullptr;
      if constexpr (KSP) {
#pragma unroll
        for (int q = 0; q < PX; ++q) cids[q] = jmin[q];
      } else {
        unstash(0, c, cids);
      }
      static_steps<0, PX, RB>([&](auto qc) { refine_batch(qc, cids, vmin, wres_min, co, wl, ridx); });
      store_row<PX>(idx_min + cb_off, lane_ob, ridx, first_qs);
      if (y_min) store_row<PX>(y_min + cb_off, lane_ob, vmin, first_qs);
    }
    if (DO_MAX) {
      if (wrps > 0 && s_max % wrps == 0 && !(DO_MIN && NT == 1)) stage_rows(s_max);
      const float* wl = wrps > 0 ? wstage + (s_max % wrps) * KS : nullptr;
      if constexpr (KSP) {
#pragma unroll
        for (int q = 0; q < PX; ++q) cids[q] = jmax[q];
      } else {
        unstash(NBR - 1, c, cids);
      }
      static_steps<0, PX, RB>([&](auto qc) { refine_batch(qc, cids, vmax, wres_max, co, wl, ridx); });
      store_row<PX>(idx_max + cb_off, lane_ob, ridx, first_qs);
      if (y_max) store_row<PX>(y_max + cb_off, lane_ob, vmax, first_qs);
    }
#pragma unroll
    for (int q = 0; q < PX; ++q) {
      if (!DO_MIN) out[q] = vmax[q];
      else if (!DO_MAX) out[q] = vmin[q];
      else out[q] = combine(ca, vmin[q], cb, vmax[q]);
    }
    // the layer's epilogue on the combined output: bias, folded batch norm, residual (wave-uniform branches)
    if (ep.bias) {
      const float bv = ep.bias[co];
#pragma unroll
      for (int q = 0; q < PX; ++q) out[q] = __fadd_rn(out[q], bv);
    }
    if (ep.scale) {
      const float sc = ep.scale[co], sf = ep.shift ? ep.shift[co] : 0.0f;
#pragma unroll
      for (int q = 0; q < PX; ++q) out[q] = __fadd_rn(__fmul_rn(out[q], sc), sf);
    }
    if (ep.residual) {
      const TO* rp = (const TO*)ep.residual + ob;
#pragma unroll
      for (int q = 0; q < PX; ++q)
        if (q >= first_qs) out[q] = __fadd_rn(out[q], ld_f32(rp, (size_t)q));
    }
    store_row<PX>(y + cb_off, lane_ob, out, first_qs);
  };
  if constexpr (KSP) {
    finish_channel(0, co0 + wave, fmin, fmax);
  } else {
#pragma unroll
    for (int c = 0; c < TN; ++c) {
      if (co0 + c >= p.C_out) break;  // wave-uniform
      finish_channel(c, co0 + c, bmin[c], bmax[c]);
    }
  }
}

// kernel rows a wave stages in LDS for the epilogue gathers: as many (a power of two) as fit its share of what the
// workgroup has left (12 KB without a staged input region: 32 KB of static LDS + 4 x 12 KB)
template <int MODE, int TN>
int staged_rows(const Params& p, long long bytes_per_wave) {
  constexpr int NT = (MODE == TCONV_PARALLEL) ? 2 : 1;
  const long long KS = (p.K + 3) & ~3;
  for (int r = TN * NT; r >= 1; r >>= 1)
    if (r * KS * 4 <= bytes_per_wave) return r;
  return 0;
}

template <int MODE, int S, int D, int TN, bool PZ, typename TO, bool XA = false, bool KSP = false>
hipError_t launch_tn(const Params& p, const void* x, const float* w_min, const float* w_max,
                     const FwdArgs& a, hipStream_t s) {
  constexpr int PX = (S == 1) ? 8 : 4;
  const int segs = (p.Wo + PX - 1) / PX;
  const long long n_units = (long long)p.N * p.Ho * segs;
  const int n_groups = (p.C_out + TN - 1) / TN;
  const long long ublocks = (n_units + 63) / 64;
  const long long gblocks = KSP ? n_groups : (n_groups + WAVES - 1) / WAVES;
  const long long blocks = ublocks * gblocks;
  if (blocks > 0x7ffffff0LL) return hipErrorInvalidValue;
#ifdef TCONV_TUNING
  // Timing experiments only, never in the default build: bit 0 skips the tap recovery, bit 1 the main loop (both give
  // WRONG results), bit 4 gathers kernel values from global memory, bit 5 forces the round-robin order.
  const char* e = getenv("TCONV_DEBUG_FLAGS");
  const int dbg = e ? atoi(e) : 0;
#else
  constexpr int dbg = 0;
#endif
  constexpr int NT = (MODE == TCONV_PARALLEL) ? 2 : 1;
  const int KS = (p.K + 3) & ~3;
  // KSP: a wave finishes one output channel; 16 KB of parked winners and 32 KB of exchanged extrema are static
  int wrps = KSP ? staged_rows<MODE, 1>(p, 8 * 1024) : staged_rows<MODE, TN>(p, 12 * 1024);
  if (dbg & 16) wrps = 0;
  const size_t lds = (size_t)WAVES * wrps * KS * sizeof(float);
  // How the 8 XCDs split the work (see the kernel): more channel parts keep an XCD's share of the kernel tensors
  // small (its scalar loads stay in its L2), fewer keep the input lines from being fetched by every XCD.  Measured
  // with one part (every XCD walks all channel blocks): +4 to +9 % and 6 to 20 times fewer bytes fetched while the
  // kernels are small next to an L2 (0.15 - 0.6 MB), -4 % to +1 % at 2.4 MB, -5 % at 4.7 MB; so the kernel tensors
  // are cut into parts of at most 1.5 MB.  TCONV_FWD_XSPLIT=1|2|4|8 fixes the number of parts (tuning aid).
  const long long w_bytes = (long long)p.C_out * p.K * (long long)sizeof(float) * NT;
  int xsplit = 1;
  while (xsplit < 8 && w_bytes / xsplit > 1536LL * 1024 && 2 * xsplit <= gblocks) xsplit *= 2;
  if (const char* ex = getenv("TCONV_FWD_XSPLIT")) {
    const int v = atoi(ex);
    if ((v == 1 || v == 2 || v == 4 || v == 8) && v <= gblocks) xsplit = v;
  }
  const int flags = dbg;
  const long long gb_per = (gblocks + xsplit - 1) / xsplit, ub_per = (ublocks + 8 / xsplit - 1) / (8 / xsplit);
  const long long grid = (dbg & FLAG_ROUND_ROBIN) ? blocks : 8 * gb_per * ub_per;
  if (grid > 0x7ffffff0LL) return hipErrorInvalidValue;
  const Epilogue ep = {a.bias, a.scale, a.shift, a.residual};
  hipLaunchKernelGGL((fwd_tiled3x3_kernel<MODE, S, D, TN, PZ, TO, XA, KSP>), dim3((unsigned)grid), dim3(WAVES * 64),
                     lds, s, p, (const TO*)x, w_min, w_max, a.alpha, a.beta, (TO*)a.y, (TO*)a.y_min, (TO*)a.y_max,
                     a.idx_min, a.idx_max, ep, segs, (int)n_units, n_groups, wrps, flags, (int)ublocks, xsplit);
  return hipGetLastError();
}

}  // namespace
}  // namespace tconv
