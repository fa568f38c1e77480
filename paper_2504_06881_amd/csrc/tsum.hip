// Sum-channel tropical convolution layers on gfx950 (fp32).
//
// Operators.  Base operators of paper Sec. 3.1 for one input channel: MinPlus2d / MaxPlus2d = the
// minimum / maximum of x + w over the KH x KW window.  Layers (i) MinPlus-Sum-Conv2d and (ii)
// MaxPlus-Sum-Conv2d sum the base operator over c_in; the two-parameter compound and parallel layers
// (Sec. 3.5, 3.6) compute
//   y[n, c_out, oh, ow] = sum over c_in of ( alpha[c_in, c_out] * MinPlus2d(x, W1) + beta[c_in, c_out] * MaxPlus2d(x, W2) ),
// W1 == W2 in the compound layer.  Padded taps are skipped (they hold the semiring identity), window
// ties keep the lowest tap, every x + w is one rounded fp32 add, a channel's term is
// fl(fl(alpha*m) + fl(beta*M)) and the channel sum adds the terms in ascending c_in starting from +0,
// each add rounded to fp32: the result does not depend on how the work is tiled.
//
// Forward: a tiled kernel for 3x3 / stride 1 (lane = 8 pixels of a row x 4 output channels, kernel
// values and coefficients wave-uniform in SGPRs, input rows in registers, NaN as padding; no
// winner is tracked, so there is no epilogue) and a one-thread-per-output kernel for everything else.
// Backward re-computes the window winners instead of storing C_in times larger index tensors:
//   sum_bwd_fused3x3_kernel  3x3 windows, all gradients of a call from ONE winner search: workgroup = (image,
//                      input channel[, band of rows]) with the grad_x plane and replicated tap bins in LDS;
//   sum_bwd_x_kernel / sum_bwd_x3x3_kernel   grad_x alone (or other windows): the same workgroup layout, every
//                      (c_out, output pixel) adds its gradient at the winner's pixel of the fp64 plane in LDS;
//   sum_bwd_w3x3_blk_kernel / sum_bwd_w_kernel   the parameter gradients alone (or other windows): workgroup =
//                      (c_in, block of c_out | one c_out[, slice of the batch]), tap bins per branch in LDS.
// What bounds the backward pass: an item (pixel, c_out, c_in) costs about 70 vector instructions (9 adds, two winner
// searches of 19, the fp64 products) and one ds_add_f64 per branch and gradient; an LDS fp64 atomic takes a compute
// unit about 22 clocks per wave, as much as 5 vector instructions, so the fused kernel (4 atomics per item) is bound
// by the LDS atomics and the separate kernels (2 each, the search done twice) by instruction issue.
#include <stdlib.h>
#include <string.h>

#include "tile_common.h"

namespace tconv {
namespace {

using namespace tile;

__device__ __forceinline__ float coef_of(const float* a, int c, int co, int C_out) {
  return a ? a[(size_t)c * C_out + co] : 1.0f;
}

// ------------------------------------------------------------------ forward, any geometry
template <int MODE>
__global__ __launch_bounds__(256) void sum_fwd_generic_kernel(Params p, const float* __restrict__ x,
                                                              const float* __restrict__ w_min,
                                                              const float* __restrict__ w_max,
                                                              const float* __restrict__ alpha,
                                                              const float* __restrict__ beta,
                                                              float* __restrict__ y) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr bool TWO = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  const size_t total = (size_t)p.N * p.C_out * p.Ho * p.Wo;
  const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= total) return;
  const int ow = (int)(o % p.Wo);
  const int oh = (int)((o / p.Wo) % p.Ho);
  const int co = (int)((o / ((size_t)p.Wo * p.Ho)) % p.C_out);
  const int n = (int)(o / ((size_t)p.Wo * p.Ho * p.C_out));
  const int KK = p.KH * p.KW;
  const int ih0 = oh * p.sh - p.ph, iw0 = ow * p.sw - p.pw;
  float acc = 0.0f;
  for (int c = 0; c < p.C_in; ++c) {
    const float* xc = x + ((size_t)n * p.C_in + c) * p.H * p.W;
    const float* wa = DO_MIN ? w_min + ((size_t)co * p.C_in + c) * KK : nullptr;
    const float* wb = DO_MAX ? w_max + ((size_t)co * p.C_in + c) * KK : nullptr;
    float m = INFINITY, M = -INFINITY;
    for (int i = 0; i < p.KH; ++i) {
      const int ih = ih0 + i * p.dh;
      if (ih < 0 || ih >= p.H) continue;
      for (int j = 0; j < p.KW; ++j) {
        const int iw = iw0 + j * p.dw;
        if (iw < 0 || iw >= p.W) continue;
        const float xv = xc[(size_t)ih * p.W + iw];
        if (DO_MIN) m = fminf(m, __fadd_rn(xv, wa[i * p.KW + j]));
        if (DO_MAX) M = fmaxf(M, __fadd_rn(xv, wb[i * p.KW + j]));
      }
    }
    float term;
    if (TWO) term = combine(coef_of(alpha, c, co, p.C_out), m, coef_of(beta, c, co, p.C_out), M);
    else term = DO_MIN ? m : M;
    acc = __fadd_rn(acc, term);
  }
  y[o] = acc;
}

// ------------------------------------------------------------------ forward, 3x3 stride 1
// Lane = PX consecutive output pixels of a row x TN output channels; wave = 64 such segments; the
// WAVES waves of a workgroup share the segments and differ in output-channel group.  Per input
// channel a lane holds 3 rows x (PX + 2*D) input values (loaded one channel ahead into a second set
// of registers), padding replaced by NaN, which v_max3 / v_min3 ignore.
template <int MODE, int D, int S, typename TO, int TN, int PX>
__global__ __launch_bounds__(WAVES * 64, (D == 1 && MODE != TCONV_PARALLEL) ? 4 : 2) void sum_fwd_tiled3x3_kernel(
    Params p, const TO* __restrict__ x, const float* __restrict__ w_min,
    const float* __restrict__ w_max, const float* __restrict__ alpha, const float* __restrict__ beta,
    TO* __restrict__ y, int segs, int n_units, int n_groups, int n_blocks, int xcd_runs, int wpb) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr bool TWO = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  // PX outputs per lane: 8 at stride 1 (4 on layers with too few lanes otherwise), 4 at stride 2
  constexpr int CORE = PX * S;                  // columns of the run every row is loaded with (32 or 16 bytes)
  constexpr int NHR = (PX - 1) * S + D + 1 - CORE;  // halo columns right of the run: D at stride 1, none at stride 2
  constexpr int XR = D + CORE + NHR;
  static_assert(NHR >= 0 && (S == 1 || (D == 1 && PX == 4)) && (PX == 4 || PX == 8),
                "geometries: stride 1 with dilation 1 or 2, stride 2 with dilation 1 and 4 outputs per lane");

  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  xcd_runs: every XCD gets a contiguous
  // run of workgroup numbers, so that the output-channel groups of a pixel block (consecutive numbers, same
  // input lines) meet in one L2.  The grid is padded to a multiple of 8; the kernel has no barrier.
  const int per_xcd = (n_blocks + 7) >> 3;
  const int bid = xcd_runs ? (int)(blockIdx.x & 7u) * per_xcd + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
  if (bid >= n_blocks) return;
  const int gblocks = (n_groups + wpb - 1) / wpb;  // wpb waves per workgroup, each a different c_out group
  const int ublock = bid / gblocks;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int group = (bid - ublock * gblocks) * wpb + wave;
  if (group >= n_groups) return;  // whole wave leaves; the kernel has no barrier
  const int co0 = group * TN;
  const int lane = threadIdx.x & 63;
  const int unit_raw = ublock * 64 + lane;
  const bool unit_ok = unit_raw < n_units;
  const int unit = unit_ok ? unit_raw : n_units - 1;
  const int seg = unit % segs;
  const int oh = (unit / segs) % p.Ho;
  const int n = unit / (segs * p.Ho);
  // the last segment of a row is shifted left so that every lane owns PX real pixels
  const int ow_nom = seg * PX;
  const int ow0 = min(ow_nom, p.Wo - PX);
  const int first_q = unit_ok ? ow_nom - ow0 : PX;

  const int iw0 = ow0 * S - p.pw;  // input column of register column 0
  const size_t HW = (size_t)p.H * p.W;
  const unsigned HWb = (unsigned)(HW * sizeof(TO));
  const rsrc_t xres = make_rsrc(x, (unsigned)((size_t)p.N * p.C_in * HW * sizeof(TO)));
  unsigned roff[3], mrow[3];
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int ih = oh * S - p.ph + i * D;
    mrow[i] = (ih >= 0 && ih < p.H) ? 0u : 0xffffffffu;
    const int ihc = min(max(ih, 0), p.H - 1);
    // byte offset of the first core column (iw0 + D >= 0 because pad_w <= D)
    roff[i] = (unsigned)(((size_t)n * p.C_in * HW + (size_t)ihc * p.W + (size_t)(iw0 + D)) * sizeof(TO));
  }
  // halo columns: D left of the run, NHR right of it; at stride 2 the run's last column can lie past the row end
  // (the load then takes the next row's first value, or 0 past the tensor), so every column has a mask
  int hoff[D + NHR];
  unsigned mcol[XR];
#pragma unroll
  for (int o = 0; o < XR; ++o) {
    const int iw = iw0 + o;
    mcol[o] = (iw >= 0 && iw < p.W) ? 0u : 0xffffffffu;
  }
#pragma unroll
  for (int h = 0; h < D + NHR; ++h) {
    const int o = (h < D) ? h : h + CORE;
    hoff[h] = (min(max(iw0 + o, 0), p.W - 1) - (iw0 + D)) * (int)sizeof(TO);
  }
  auto load_rows = [&](float (&xs)[3][XR], int c) {
    const unsigned soff = (unsigned)min(c, p.C_in - 1) * HWb;
#pragma unroll
    for (int i = 0; i < 3; ++i) {
#pragma unroll
      for (int h = 0; h < D; ++h) xs[i][h] = load_one<TO>(xres, roff[i] + (unsigned)hoff[h], soff);
      load_run<CORE, TO>(&xs[i][D], xres, roff[i], soff);
#pragma unroll
      for (int h = 0; h < NHR; ++h) xs[i][D + CORE + h] = load_one<TO>(xres, roff[i] + (unsigned)hoff[D + h], soff);
    }
  };
  auto mask_rows = [&](float (&xs)[3][XR]) {
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
      for (int o = 0; o < XR; ++o) {
        const bool inside = S == 1 && o >= D && o < D + CORE;  // stride 1: the run lies inside the row
        xs[i][o] = nan_or(xs[i][o], inside ? mrow[i] : (mrow[i] | mcol[o]));
      }
  };

  float acc[TN][PX];
#pragma unroll
  for (int c = 0; c < TN; ++c)
#pragma unroll
    for (int q = 0; q < PX; ++q) acc[c][q] = 0.0f;

  // one input channel: for every output channel of the lane the 9 kernel values (and the two
  // coefficients) are wave-uniform scalars; 9 adds, 4 + 4 three-operand extrema, the rounded combine
  auto channel = [&](const float (&xs)[3][XR], int c) {
#pragma unroll
    for (int t = 0; t < TN; ++t) {
      const int co = min(co0 + t, p.C_out - 1);
      const float* wa = DO_MIN ? w_min + ((size_t)co * p.C_in + c) * 9 : nullptr;
      const float* wb = DO_MAX ? w_max + ((size_t)co * p.C_in + c) * 9 : nullptr;
      float ka[9], kb[9];
#pragma unroll
      for (int k = 0; k < 9; ++k) {
        if (DO_MIN) ka[k] = wa[k];
        if (DO_MAX) kb[k] = wb[k];
      }
      const float ca = TWO ? coef_of(alpha, c, co, p.C_out) : 1.0f;
      const float cb = TWO ? coef_of(beta, c, co, p.C_out) : 1.0f;
#pragma unroll
      for (int q = 0; q < PX; ++q) {
        float sa[9], sb[9];
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
          for (int j = 0; j < 3; ++j) {
            const float xv = xs[i][q * S + j * D];
            if (DO_MIN) sa[i * 3 + j] = __fadd_rn(xv, ka[i * 3 + j]);
            if (DO_MAX) sb[i * 3 + j] = (MODE == TCONV_COMPOUND) ? sa[i * 3 + j] : __fadd_rn(xv, kb[i * 3 + j]);
          }
        float m = 0.f, M = 0.f;
        if (DO_MIN) {
          m = fminf(fminf(sa[0], sa[1]), sa[2]);
          m = fminf(fminf(m, sa[3]), sa[4]);
          m = fminf(fminf(m, sa[5]), sa[6]);
          m = fminf(fminf(m, sa[7]), sa[8]);
        }
        if (DO_MAX) {
          M = fmaxf(fmaxf(sb[0], sb[1]), sb[2]);
          M = fmaxf(fmaxf(M, sb[3]), sb[4]);
          M = fmaxf(fmaxf(M, sb[5]), sb[6]);
          M = fmaxf(fmaxf(M, sb[7]), sb[8]);
        }
        const float term = TWO ? combine(ca, m, cb, M) : (DO_MIN ? m : M);
        acc[t][q] = __fadd_rn(acc[t][q], term);
      }
    }
  };

  float xa[3][XR], xb[3][XR];
  load_rows(xa, 0);
  for (int c = 0; c < p.C_in; c += 2) {
    load_rows(xb, c + 1);  // past the last channel: a clamped, unused reload
    mask_rows(xa);
    channel(xa, c);
    if (c + 1 < p.C_in) {  // wave-uniform
      load_rows(xa, c + 2);
      mask_rows(xb);
      channel(xb, c + 1);
    }
  }

  const size_t plane = (size_t)p.Ho * p.Wo;
#pragma unroll
  for (int t = 0; t < TN; ++t) {
    const int co = co0 + t;
    if (co >= p.C_out) break;  // wave-uniform
    store_row<PX>(y + ((size_t)n * p.C_out + co) * plane + (size_t)oh * p.Wo + ow0, acc[t], first_q);
  }
}

// ------------------------------------------------------------------ backward
// Window of one (c_out, c_in, output pixel): the 9 (KH*KW) sums are scanned in ascending tap order with
// strict compares, so ties keep the lowest tap.  px points at the channel's H x W plane (global or LDS,
// row stride `rs`, first row `row0`).
struct Winner {
  float v;
  int ih, iw, t;
};
template <bool WANT_MAX>
__device__ __forceinline__ Winner scan_window(const Params& p, const float* px, int rs, int row0,
                                              const float* __restrict__ w9, int oh, int ow) {
  Winner r = {WANT_MAX ? -INFINITY : INFINITY, 0, 0, -1};
  const int ih0 = oh * p.sh - p.ph, iw0 = ow * p.sw - p.pw;
  for (int i = 0; i < p.KH; ++i) {
    const int ih = ih0 + i * p.dh;
    if (ih < 0 || ih >= p.H) continue;
    for (int j = 0; j < p.KW; ++j) {
      const int iw = iw0 + j * p.dw;
      if (iw < 0 || iw >= p.W) continue;
      const float s = __fadd_rn(px[(ih - row0) * rs + iw], w9[i * p.KW + j]);
      if (r.t < 0 || (WANT_MAX ? (s > r.v) : (s < r.v))) { r.v = s; r.ih = ih; r.iw = iw; r.t = i * p.KW + j; }
    }
  }
  return r;
}

// grad_x.  Workgroup = (image n, input channel c, band of input rows [r0, r0 + TH)): the band of the
// grad_x plane lives in LDS as fp64 next to the input rows the windows that can reach it read
// (fp32); every (c_out, output pixel whose window can reach the band) re-computes its winners and adds
// coef * gy at the winner's pixel if that lies in the band; the band is then written with plain stores.
template <int MODE>
__global__ __launch_bounds__(256) void sum_bwd_x_kernel(Params p, const float* __restrict__ x,
                                                        const float* __restrict__ w_min,
                                                        const float* __restrict__ w_max,
                                                        const float* __restrict__ alpha,
                                                        const float* __restrict__ beta,
                                                        const float* __restrict__ gy,
                                                        float* __restrict__ grad_x, int TH, int n_bands) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr bool TWO = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  extern __shared__ double lds_d[];
  const int band = blockIdx.x % n_bands;
  const int c = (blockIdx.x / n_bands) % p.C_in;
  const int n = blockIdx.x / (n_bands * p.C_in);
  const int r0 = band * TH, r1 = min(r0 + TH, p.H);
  const int eh = p.dh * (p.KH - 1);
  // output rows whose window [oh*sh - ph, oh*sh - ph + eh] meets [r0, r1)
  const int oh_lo = max(0, (r0 + p.ph - eh + p.sh - 1) / p.sh);
  const int oh_hi = min(p.Ho - 1, (r1 - 1 + p.ph) / p.sh);
  // input rows those windows read
  const int xr0 = max(0, oh_lo * p.sh - p.ph), xr1 = min(p.H, oh_hi * p.sh - p.ph + eh + 1);
  double* const tile = lds_d;                                   // [(r1 - r0) x W]
  float* const xs = (float*)(lds_d + (size_t)TH * p.W);         // [(xr1 - xr0) x W]
  for (int i = threadIdx.x; i < (r1 - r0) * p.W; i += blockDim.x) tile[i] = 0.0;
  const float* xc = x + ((size_t)n * p.C_in + c) * p.H * p.W;
  if (oh_hi >= oh_lo)
    for (int i = threadIdx.x; i < (xr1 - xr0) * p.W; i += blockDim.x) xs[i] = xc[(size_t)xr0 * p.W + i];
  __syncthreads();
  const int rows = max(oh_hi - oh_lo + 1, 0);
  const int per_co = rows * p.Wo;
  const int KK = p.KH * p.KW;
  for (int it = threadIdx.x; it < per_co * p.C_out; it += blockDim.x) {
    const int co = it / per_co;
    const int rem = it - co * per_co;
    const int oh = oh_lo + rem / p.Wo, ow = rem % p.Wo;
    const float g = gy[(((size_t)n * p.C_out + co) * p.Ho + oh) * p.Wo + ow];
    if (DO_MIN) {
      const Winner wv = scan_window<false>(p, xs, p.W, xr0, w_min + ((size_t)co * p.C_in + c) * KK, oh, ow);
      if (wv.ih >= r0 && wv.ih < r1)
        atomicAdd(&tile[(wv.ih - r0) * p.W + wv.iw], (double)(TWO ? coef_of(alpha, c, co, p.C_out) : 1.0f) * (double)g);
    }
    if (DO_MAX) {
      const Winner wv = scan_window<true>(p, xs, p.W, xr0, w_max + ((size_t)co * p.C_in + c) * KK, oh, ow);
      if (wv.ih >= r0 && wv.ih < r1)
        atomicAdd(&tile[(wv.ih - r0) * p.W + wv.iw], (double)(TWO ? coef_of(beta, c, co, p.C_out) : 1.0f) * (double)g);
    }
  }
  __syncthreads();
  float* gxc = grad_x + ((size_t)n * p.C_in + c) * p.H * p.W + (size_t)r0 * p.W;
  for (int i = threadIdx.x; i < (r1 - r0) * p.W; i += blockDim.x) gxc[i] = (float)tile[i];
}

// Extremum of the 9 sums of a 3 x 3 window and its lowest tap, without a compare-and-select chain over the taps:
// three v_min3 / v_max3 over the rows, one over the row results, then the first row and the first column of it
// that equal the extremum (19 instructions where the chain takes 27).  NaN sums (taps outside the image) are
// ignored by the three-operand instructions and equal nothing.
template <bool WANT_MAX>
__device__ __forceinline__ void window_extremum9_rc(const float (&s)[9], float& best, int& row, int& col) {
  float r[3];
#pragma unroll
  for (int i = 0; i < 3; ++i)
    r[i] = WANT_MAX ? fmaxf(fmaxf(s[3 * i], s[3 * i + 1]), s[3 * i + 2]) : fminf(fminf(s[3 * i], s[3 * i + 1]), s[3 * i + 2]);
  best = WANT_MAX ? fmaxf(fmaxf(r[0], r[1]), r[2]) : fminf(fminf(r[0], r[1]), r[2]);
  const bool c0 = r[0] == best, c1 = r[1] == best;
  row = c0 ? 0 : (c1 ? 1 : 2);
  const float a0 = c0 ? s[0] : (c1 ? s[3] : s[6]);
  const float a1 = c0 ? s[1] : (c1 ? s[4] : s[7]);
  col = (a0 == best) ? 0 : ((a1 == best) ? 1 : 2);
}
template <bool WANT_MAX>
__device__ __forceinline__ void window_extremum9(const float (&s)[9], float& best, int& tap) {
  float r[3];
#pragma unroll
  for (int i = 0; i < 3; ++i)
    r[i] = WANT_MAX ? fmaxf(fmaxf(s[3 * i], s[3 * i + 1]), s[3 * i + 2]) : fminf(fminf(s[3 * i], s[3 * i + 1]), s[3 * i + 2]);
  best = WANT_MAX ? fmaxf(fmaxf(r[0], r[1]), r[2]) : fminf(fminf(r[0], r[1]), r[2]);
  const bool c0 = r[0] == best, c1 = r[1] == best;
  const int row = c0 ? 0 : (c1 ? 1 : 2);
  const float a0 = c0 ? s[0] : (c1 ? s[3] : s[6]);
  const float a1 = c0 ? s[1] : (c1 ? s[4] : s[7]);
  const int col = (a0 == best) ? 0 : ((a1 == best) ? 1 : 2);
  tap = row * 3 + col;
}

// grad_x for 3x3 windows: the same workgroup layout, but a thread keeps the 9 input values of its output
// pixel in registers and walks all output channels with them (the kernel values of a (c_out, c_in)
// pair are wave-uniform scalars, gy is read coalesced), so that a (pixel, c_out) item costs about 70
// vector instructions and one LDS atomic per branch.
template <int MODE>
__global__ __launch_bounds__(256) void sum_bwd_x3x3_kernel(Params p, const float* __restrict__ x,
                                                           const float* __restrict__ w_min,
                                                           const float* __restrict__ w_max,
                                                           const float* __restrict__ alpha,
                                                           const float* __restrict__ beta,
                                                           const float* __restrict__ gy,
                                                           float* __restrict__ grad_x, int TH, int n_bands) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr bool TWO = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  extern __shared__ double lds_d[];
  const int band = blockIdx.x % n_bands;
  const int c = (blockIdx.x / n_bands) % p.C_in;
  const int n = blockIdx.x / (n_bands * p.C_in);
  const int r0 = band * TH, r1 = min(r0 + TH, p.H);
  const int eh = 2 * p.dh;
  const int oh_lo = max(0, (r0 + p.ph - eh + p.sh - 1) / p.sh);
  const int oh_hi = min(p.Ho - 1, (r1 - 1 + p.ph) / p.sh);
  const int xr0 = max(0, oh_lo * p.sh - p.ph), xr1 = min(p.H, oh_hi * p.sh - p.ph + eh + 1);
  double* const tile = lds_d;                                   // [(r1 - r0) x W]
  float* const xs = (float*)(lds_d + (size_t)TH * p.W);         // [(xr1 - xr0) x W]
  for (int i = threadIdx.x; i < (r1 - r0) * p.W; i += blockDim.x) tile[i] = 0.0;
  const float* xc = x + ((size_t)n * p.C_in + c) * p.H * p.W;
  if (oh_hi >= oh_lo)
    for (int i = threadIdx.x; i < (xr1 - xr0) * p.W; i += blockDim.x) xs[i] = xc[(size_t)xr0 * p.W + i];
  __syncthreads();
  const int rows = max(oh_hi - oh_lo + 1, 0);
  const int n_pix = rows * p.Wo;
  const size_t plane = (size_t)p.Ho * p.Wo;
  for (int pix = threadIdx.x; pix < n_pix; pix += blockDim.x) {
    const int oh = oh_lo + pix / p.Wo, ow = pix % p.Wo;
    const int ih0 = oh * p.sh - p.ph, iw0 = ow * p.sw - p.pw;
    // the window's input values; a tap outside the image holds the identity of its branch and never wins
    float xlo[9], xhi[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) {
      const int ih = ih0 + (t / 3) * p.dh, iw = iw0 + (t % 3) * p.dw;
      const bool ok = ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
      const float v = ok ? xs[(ih - xr0) * p.W + iw] : 0.f;
      xlo[t] = ok ? v : INFINITY;
      xhi[t] = ok ? v : -INFINITY;
    }
    const float* gyp = gy + (size_t)n * p.C_out * plane + (size_t)oh * p.Wo + ow;
    for (int co = 0; co < p.C_out; ++co) {  // uniform over the workgroup
      const float g = gyp[(size_t)co * plane];
      if (DO_MIN) {
        const float* w9 = w_min + ((size_t)co * p.C_in + c) * 9;
        float sums[9], best;
        int ts;
#pragma unroll
        for (int t = 0; t < 9; ++t) sums[t] = __fadd_rn(xlo[t], w9[t]);
        window_extremum9<false>(sums, best, ts);
        const int ih = ih0 + (ts / 3) * p.dh, iw = iw0 + (ts % 3) * p.dw;
        if (ih >= r0 && ih < r1)
          atomicAdd(&tile[(ih - r0) * p.W + iw], (double)(TWO ? coef_of(alpha, c, co, p.C_out) : 1.0f) * (double)g);
      }
      if (DO_MAX) {
        const float* w9 = w_max + ((size_t)co * p.C_in + c) * 9;
        float sums[9], best;
        int ts;
#pragma unroll
        for (int t = 0; t < 9; ++t) sums[t] = __fadd_rn(xhi[t], w9[t]);
        window_extremum9<true>(sums, best, ts);
        const int ih = ih0 + (ts / 3) * p.dh, iw = iw0 + (ts % 3) * p.dw;
        if (ih >= r0 && ih < r1)
          atomicAdd(&tile[(ih - r0) * p.W + iw], (double)(TWO ? coef_of(beta, c, co, p.C_out) : 1.0f) * (double)g);
      }
    }
  }
  __syncthreads();
  float* gxc = grad_x + ((size_t)n * p.C_in + c) * p.H * p.W + (size_t)r0 * p.W;
  for (int i = threadIdx.x; i < (r1 - r0) * p.W; i += blockDim.x) gxc[i] = (float)tile[i];
}

// grad_w, grad_alpha, grad_beta.  Workgroup = (c_out, c_in, slice of the batch): each thread walks
// output pixels, re-computes the winners and keeps KK tap sums per branch (in LDS, a private column per
// thread, fp64) plus the two coefficient sums; a tree reduction over the threads, then one fp32 atomic
// per value into the zero-filled results.
template <int MODE>
__global__ __launch_bounds__(256) void sum_bwd_w_kernel(Params p, const float* __restrict__ x,
                                                        const float* __restrict__ w_min,
                                                        const float* __restrict__ w_max,
                                                        const float* __restrict__ alpha,
                                                        const float* __restrict__ beta,
                                                        const float* __restrict__ gy,
                                                        float* __restrict__ grad_w_min,
                                                        float* __restrict__ grad_w_max,
                                                        float* __restrict__ grad_alpha,
                                                        float* __restrict__ grad_beta, int n_per_block) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr bool TWO = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  constexpr int NBR = (DO_MIN && DO_MAX) ? 2 : 1;
  extern __shared__ double lds_d[];
  const int KK = p.KH * p.KW;
  const int NV = NBR * (KK + 1);  // per thread: KK tap sums and one coefficient sum per branch
  const int NT = blockDim.x;                 // 256, or fewer for large kernel windows (LDS)
  double* const mine = lds_d + threadIdx.x;  // value v of thread t at lds_d[v * NT + t]
  for (int v = 0; v < NV; ++v) mine[v * NT] = 0.0;
  const int co = blockIdx.x / p.C_in, c = blockIdx.x % p.C_in;
  const int n0 = blockIdx.y * n_per_block, n1 = min(n0 + n_per_block, p.N);
  const float* wa = DO_MIN ? w_min + ((size_t)co * p.C_in + c) * KK : nullptr;
  const float* wb = DO_MAX ? w_max + ((size_t)co * p.C_in + c) * KK : nullptr;
  const double ca = TWO ? (double)coef_of(alpha, c, co, p.C_out) : 1.0;
  const double cb = TWO ? (double)coef_of(beta, c, co, p.C_out) : 1.0;
  const int plane = p.Ho * p.Wo;
  for (int n = n0; n < n1; ++n) {
    const float* xc = x + ((size_t)n * p.C_in + c) * p.H * p.W;
    const float* gyc = gy + ((size_t)n * p.C_out + co) * plane;
    for (int i = threadIdx.x; i < plane; i += blockDim.x) {
      const int oh = i / p.Wo, ow = i % p.Wo;
      const double g = (double)gyc[i];
      if (DO_MIN) {
        const Winner wv = scan_window<false>(p, xc, p.W, 0, wa, oh, ow);
        mine[wv.t * NT] += ca * g;
        mine[KK * NT] += g * (double)wv.v;
      }
      if (DO_MAX) {
        const Winner wv = scan_window<true>(p, xc, p.W, 0, wb, oh, ow);
        const int b = (NBR - 1) * (KK + 1);
        mine[(b + wv.t) * NT] += cb * g;
        mine[(b + KK) * NT] += g * (double)wv.v;
      }
    }
  }
  __syncthreads();
  for (int h = NT / 2; h > 0; h >>= 1) {
    if ((int)threadIdx.x < h)
      for (int v = 0; v < NV; ++v) mine[v * NT] += mine[v * NT + h];
    __syncthreads();
  }
  // thread v publishes value v
  for (int v = threadIdx.x; v < NV; v += blockDim.x) {
    const int br = v / (KK + 1), k = v % (KK + 1);
    const bool is_max = DO_MAX && (NBR == 1 || br == 1);
    const float val = (float)lds_d[v * NT];
    if (k < KK) {
      float* gw = is_max ? grad_w_max : grad_w_min;
      if (gw) atomicAdd(gw + ((size_t)co * p.C_in + c) * KK + k, val);
    } else if (TWO) {
      float* gc = is_max ? grad_beta : grad_alpha;
      if (gc) atomicAdd(gc + (size_t)c * p.C_out + co, val);
    }
  }
}

// grad_w, grad_alpha, grad_beta for 3x3 windows, several output channels per workgroup.  Workgroup = (input channel c,
// block of CB output channels, slice of the batch).  A thread takes output pixels; per pixel it works out the tap
// addresses and loads the 9 input values ONCE and then walks the CB output channels with them (kernel values and
// coefficients are wave-uniform scalars, gy is read coalesced): the address arithmetic and the loads, more than half
// of the one-channel kernel's instructions, are shared by CB items.  The tap sums go to LDS bins [REP][CB][branch][9]
// of fp64 with ds_add_f64; a lane uses replica (lane mod REP), so that at most 64 / REP lanes of a wave can meet in
// one bin.  The coefficient sums stay in fp64 registers.  At the end the replicas are added in a fixed order and each
// value goes into the zero-filled result with one fp32 atomic.
constexpr int SUMW_CB = 4, SUMW_REP = 16;
template <int MODE>
__global__ __launch_bounds__(256) void sum_bwd_w3x3_blk_kernel(Params p, const float* __restrict__ x,
                                                               const float* __restrict__ w_min,
                                                               const float* __restrict__ w_max,
                                                               const float* __restrict__ alpha,
                                                               const float* __restrict__ beta,
                                                               const float* __restrict__ gy,
                                                               float* __restrict__ grad_w_min,
                                                               float* __restrict__ grad_w_max,
                                                               float* __restrict__ grad_alpha,
                                                               float* __restrict__ grad_beta, int n_per_block,
                                                               int n_coblocks) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr bool TWO = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  constexpr int NBR = (DO_MIN && DO_MAX) ? 2 : 1;
  constexpr int CB = SUMW_CB, REP = SUMW_REP;
  __shared__ double bins[CB][NBR][REP][11];  // 11: an odd stride spreads the replicas over the LDS banks
  __shared__ double csum[4][CB][2];  // per wave: coefficient sums
  for (int e = threadIdx.x; e < CB * NBR * REP * 11; e += blockDim.x) (&bins[0][0][0][0])[e] = 0.0;
  const int c = blockIdx.x / n_coblocks, cob = blockIdx.x - c * n_coblocks;
  const int co0 = cob * CB;
  const int n0 = blockIdx.y * n_per_block, n1 = min(n0 + n_per_block, p.N);
  const int plane = p.Ho * p.Wo;
  const rsrc_t xres = make_rsrc(x, (unsigned)((size_t)p.N * p.C_in * p.H * p.W * sizeof(float)));
  const int oh_first = (int)threadIdx.x / p.Wo, ow_first = (int)threadIdx.x % p.Wo;
  const int d_oh = (int)blockDim.x / p.Wo, d_ow = (int)blockDim.x % p.Wo;
  const int myrep = threadIdx.x & (REP - 1);
  double sa[CB], sb[CB];
#pragma unroll
  for (int b = 0; b < CB; ++b) { sa[b] = 0.0; sb[b] = 0.0; }
  __syncthreads();
  for (int n = n0; n < n1; ++n) {
    const unsigned xbase = (unsigned)(((size_t)n * p.C_in + c) * p.H * p.W * sizeof(float));  // uniform
    int oh = oh_first, ow = ow_first;
    for (int i = threadIdx.x; i < plane; i += blockDim.x, oh += d_oh, ow += d_ow) {
      if (ow >= p.Wo) { ow -= p.Wo; ++oh; }
      const int ih0 = oh * p.sh - p.ph, iw0 = ow * p.sw - p.pw;
      unsigned roff[3], coff[3];
      bool rok[3], cok[3];
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        const int ih = ih0 + k * p.dh, iw = iw0 + k * p.dw;
        rok[k] = ih >= 0 && ih < p.H;
        cok[k] = iw >= 0 && iw < p.W;
        roff[k] = (unsigned)(min(max(ih, 0), p.H - 1) * p.W) * 4u;
        coff[k] = (unsigned)min(max(iw, 0), p.W - 1) * 4u;
      }
      float xv[9];
#pragma unroll
      for (int t = 0; t < 9; ++t) xv[t] = load_one<float>(xres, roff[t / 3] + coff[t % 3], xbase);
#pragma unroll
      for (int t = 0; t < 9; ++t)  // a tap outside the image becomes NaN once for both branches: never the extremum
        xv[t] = (rok[t / 3] && cok[t % 3]) ? xv[t] : __uint_as_float(0x7fc00000u);
#pragma unroll
      for (int b = 0; b < CB; ++b) {
        const int co = min(co0 + b, p.C_out - 1);  // a block past C_out repeats the last channel and publishes nothing
        const float* ka = DO_MIN ? w_min + ((size_t)co * p.C_in + c) * 9 : nullptr;
        const float* kb = DO_MAX ? w_max + ((size_t)co * p.C_in + c) * 9 : nullptr;
        const double g = (double)gy[((size_t)n * p.C_out + co) * plane + i];
        float s1[9], s2[9];
#pragma unroll
        for (int t = 0; t < 9; ++t) {
          if (DO_MIN) s1[t] = __fadd_rn(xv[t], ka[t]);
          if (DO_MAX) s2[t] = (MODE == TCONV_COMPOUND) ? s1[t] : __fadd_rn(xv[t], kb[t]);
        }
        if (DO_MIN) {
          float bmin; int tmin;
          window_extremum9<false>(s1, bmin, tmin);
          const double ca = TWO ? (double)coef_of(alpha, c, co, p.C_out) : 1.0;
          atomicAdd(&bins[b][0][myrep][tmin], ca * g);
          sa[b] += g * (double)bmin;
        }
        if (DO_MAX) {
          float bmax; int tmax;
          window_extremum9<true>(s2, bmax, tmax);
          const double cb = TWO ? (double)coef_of(beta, c, co, p.C_out) : 1.0;
          atomicAdd(&bins[b][NBR - 1][myrep][tmax], cb * g);
          sb[b] += g * (double)bmax;
        }
      }
    }
  }
  // coefficient sums: lanes of a wave by shuffles (fixed tree), then the four waves in order
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int b = 0; b < CB; ++b) {
    double va = sa[b], vb = sb[b];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      va += __shfl_down(va, off, 64);
      vb += __shfl_down(vb, off, 64);
    }
    if (lane == 0) { csum[wave][b][0] = va; csum[wave][b][1] = vb; }
  }
  __syncthreads();
  for (int v = threadIdx.x; v < CB * NBR * 9; v += blockDim.x) {
    const int b = v / (NBR * 9), r = v - b * (NBR * 9), br = r / 9, t = r - br * 9;
    if (co0 + b >= p.C_out) continue;
    double sum = 0.0;
#pragma unroll
    for (int q = 0; q < REP; ++q) sum += bins[b][br][q][t];
    const bool is_max = DO_MAX && (NBR == 1 || br == 1);
    float* gw = is_max ? grad_w_max : grad_w_min;
    if (gw) atomicAdd(gw + ((size_t)(co0 + b) * p.C_in + c) * 9 + t, (float)sum);
  }
  if (TWO && threadIdx.x < CB * 2) {
    const int b = threadIdx.x >> 1, which = threadIdx.x & 1;
    if (co0 + b < p.C_out) {
      const double sum = csum[0][b][which] + csum[1][b][which] + csum[2][b][which] + csum[3][b][which];
      float* gc = which ? grad_beta : grad_alpha;
      if (gc) atomicAdd(gc + (size_t)c * p.C_out + (co0 + b), (float)sum);
    }
  }
}

// All gradients of a 3x3 layer from ONE winner search.  Workgroup = (image n, input channel c, band of input rows), as
// in the grad_x kernel above: the band of the grad_x plane (fp64) and the input rows its windows read (fp32) live in
// LDS.  A thread keeps the 9 input values of up to PT of its output pixels in registers and walks the output channels
// (kernel values and coefficients are wave-uniform scalars, gy is read coalesced).  Per (pixel, c_out) item: 9 adds
// (shared by both branches in compound mode), the two winner searches, and from their result
//   grad_x:      one ds_add_f64 per branch at the winner's pixel of the band,
//   grad_w:      one ds_add_f64 per branch into LDS bins [COB][branch][REP][11] (a lane uses replica lane mod REP; the
//                odd stride of 11 doubles spreads the replicas over the LDS banks: with a stride that is a multiple
//                of 32 doubles every replica of a tap sits in the same bank and the adds of a wave serialise),
//   grad_alpha / grad_beta: g * extremum summed over the thread's pixels in registers, one ds_add_f64 per
//                (thread, c_out, branch) into a tenth bin.
// The output channels are walked in chunks of COB (the bins of one chunk fit the LDS next to the band); after a chunk
// the replicas are added in a fixed order and every value goes into the zero-filled result with one fp32 atomic.
// An output pixel is scanned by every band its window reaches (for grad_x) but counts for the parameter gradients only
// in the band that holds the first row of its window that lies inside the image.
// ONE_BAND: the band is the whole plane (the common case), so every winner lands in it and every scanned pixel counts
// here: the per-item range checks drop out.
constexpr int SUMF_PT = 4, SUMF_REP = 8;
template <int MODE, bool ONE_BAND>
__global__ __launch_bounds__(256) void sum_bwd_fused3x3_kernel(Params p, const float* __restrict__ x,
                                                               const float* __restrict__ w_min,
                                                               const float* __restrict__ w_max,
                                                               const float* __restrict__ alpha,
                                                               const float* __restrict__ beta,
                                                               const float* __restrict__ gy,
                                                               float* __restrict__ grad_x,
                                                               float* __restrict__ grad_w_min,
                                                               float* __restrict__ grad_w_max,
                                                               float* __restrict__ grad_alpha,
                                                               float* __restrict__ grad_beta, int TH, int n_bands,
                                                               int COB) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr bool TWO = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  constexpr int NBR = (DO_MIN && DO_MAX) ? 2 : 1;
  constexpr int PT = SUMF_PT, REP = SUMF_REP;
  extern __shared__ double lds_d[];
  const int band = blockIdx.x % n_bands;
  const int c = (blockIdx.x / n_bands) % p.C_in;
  const int n = blockIdx.x / (n_bands * p.C_in);
  const int r0 = band * TH, r1 = min(r0 + TH, p.H);
  const int eh = 2 * p.dh;
  const int oh_lo = max(0, (r0 + p.ph - eh + p.sh - 1) / p.sh);
  const int oh_hi = min(p.Ho - 1, (r1 - 1 + p.ph) / p.sh);
  const int xr0 = max(0, oh_lo * p.sh - p.ph), xr1 = min(p.H, oh_hi * p.sh - p.ph + eh + 1);
  double* const tile = lds_d;                                           // [(r1 - r0) x W]
  double* const bins = lds_d + (size_t)TH * p.W;                        // [COB][NBR][REP][11]
  float* const xs = (float*)(bins + (size_t)COB * NBR * REP * 11);      // [(xr1 - xr0) x W]
  for (int i = threadIdx.x; i < (r1 - r0) * p.W; i += blockDim.x) tile[i] = 0.0;
  const float* xc = x + ((size_t)n * p.C_in + c) * p.H * p.W;
  if (oh_hi >= oh_lo)
    for (int i = threadIdx.x; i < (xr1 - xr0) * p.W; i += blockDim.x) xs[i] = xc[(size_t)xr0 * p.W + i];
  const int rows = max(oh_hi - oh_lo + 1, 0);
  const int n_pix = rows * p.Wo;
  const size_t plane = (size_t)p.Ho * p.Wo;
  double* const mybins = bins + (size_t)(threadIdx.x & (REP - 1)) * 11;
  const int row_step8 = p.dh * p.W * 8, col_step8 = p.dw * 8;  // byte steps of a tap row / column inside the band
  for (int cob = 0; cob < p.C_out; cob += COB) {
    const int ncb = min(COB, p.C_out - cob);
    __syncthreads();  // the previous chunk's bins have been published (first pass: tile and xs are written)
    for (int e = threadIdx.x; e < COB * NBR * REP * 11; e += blockDim.x) bins[e] = 0.0;
    __syncthreads();
    for (int base = 0; base < n_pix; base += PT * (int)blockDim.x) {
      // the thread's pixels of this round: window values (padding = NaN: never an extremum), where tap (0, 0) falls
      // in the band (byte offset, may be negative), which tap rows fall inside the band, whether the pixel counts
      // for the parameter gradients here
      float xv[PT][9];
      int t0off[PT], rowmask[PT];
      bool live[PT], own[PT];
      size_t gyoff[PT];
#pragma unroll
      for (int k = 0; k < PT; ++k) {
        const int pix = base + k * (int)blockDim.x + (int)threadIdx.x;
        live[k] = pix < n_pix;
        const int pr = live[k] ? pix / p.Wo : 0;
        const int oh = oh_lo + pr, ow = live[k] ? pix - pr * p.Wo : 0;
        const int ih0 = oh * p.sh - p.ph, iw0 = ow * p.sw - p.pw;
        rowmask[k] = 0;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
          const int ih = ih0 + (t / 3) * p.dh, iw = iw0 + (t % 3) * p.dw;
          const bool ok = ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
          xv[k][t] = ok ? xs[(ih - xr0) * p.W + iw] : __uint_as_float(0x7fc00000u);
        }
#pragma unroll
        for (int ii = 0; ii < 3; ++ii) {
          const int ih = ih0 + ii * p.dh;
          if (ih >= r0 && ih < r1) rowmask[k] |= 1 << ii;
        }
        t0off[k] = ((ih0 - r0) * p.W + iw0) * 8;
        // the first row of the window that lies inside the image (ih0 < H always): in exactly one band, and that
        // band scans this output
        const int ihv = ih0 >= 0 ? ih0 : (ih0 + p.dh >= 0 ? ih0 + p.dh : ih0 + 2 * p.dh);
        own[k] = live[k] && ihv >= r0 && ihv < r1;
        gyoff[k] = (size_t)n * p.C_out * plane + (size_t)oh * p.Wo + ow;
      }
      for (int b = 0; b < ncb; ++b) {  // uniform over the workgroup
        const int co = cob + b;
        const float* ka = DO_MIN ? w_min + ((size_t)co * p.C_in + c) * 9 : nullptr;
        const float* kb = DO_MAX ? w_max + ((size_t)co * p.C_in + c) * 9 : nullptr;
        const double ca = TWO ? (double)coef_of(alpha, c, co, p.C_out) : 1.0;
        const double cb = TWO ? (double)coef_of(beta, c, co, p.C_out) : 1.0;
        double* const bn = mybins + (size_t)b * NBR * REP * 11;
        double s_min = 0.0, s_max = 0.0;  // coefficient sums over the thread's pixels
        bool any_own = false;
#pragma unroll
        for (int k = 0; k < PT; ++k) {
          if (!live[k]) continue;
          const double g = (double)gy[gyoff[k] + (size_t)co * plane];
          float s1[9], s2[9];
#pragma unroll
          for (int t = 0; t < 9; ++t) {
            if (DO_MIN) s1[t] = __fadd_rn(xv[k][t], ka[t]);
            if (DO_MAX) s2[t] = (MODE == TCONV_COMPOUND) ? s1[t] : __fadd_rn(xv[k][t], kb[t]);
          }
          if (DO_MIN) {
            float bmin; int t;
            window_extremum9<false>(s1, bmin, t);
            const double v = ca * g;
            const int row = (t * 11) >> 5;
            if (ONE_BAND || ((rowmask[k] >> row) & 1))
              atomicAdd((double*)((char*)tile + (t0off[k] + row * row_step8 + (t - 3 * row) * col_step8)), v);
            if (ONE_BAND || own[k]) {
              atomicAdd(bn + t, v);
              s_min += g * (double)bmin;
            }
          }
          if (DO_MAX) {
            float bmax; int t;
            window_extremum9<true>(s2, bmax, t);
            const double v = cb * g;
            const int row = (t * 11) >> 5;
            if (ONE_BAND || ((rowmask[k] >> row) & 1))
              atomicAdd((double*)((char*)tile + (t0off[k] + row * row_step8 + (t - 3 * row) * col_step8)), v);
            if (ONE_BAND || own[k]) {
              atomicAdd(bn + (NBR - 1) * REP * 11 + t, v);
              s_max += g * (double)bmax;
            }
          }
          any_own = any_own || ONE_BAND || own[k];
        }
        if (TWO && any_own) {
          atomicAdd(bn + 9, s_min);
          atomicAdd(bn + REP * 11 + 9, s_max);
        }
      }
    }
    __syncthreads();
    // publish the chunk: replicas in a fixed order, one fp32 atomic per value
    for (int v = threadIdx.x; v < ncb * NBR * 10; v += blockDim.x) {
      const int b = v / (NBR * 10), r = v - b * (NBR * 10), br = r / 10, t = r - br * 10;
      double sum = 0.0;
#pragma unroll
      for (int q = 0; q < REP; ++q) sum += bins[((size_t)(b * NBR + br) * REP + q) * 11 + t];
      const bool is_max = DO_MAX && (NBR == 1 || br == 1);
      const int co = cob + b;
      if (t < 9) {
        float* gw = is_max ? grad_w_max : grad_w_min;
        if (gw) atomicAdd(gw + ((size_t)co * p.C_in + c) * 9 + t, (float)sum);
      } else if (TWO) {
        float* gc = is_max ? grad_beta : grad_alpha;
        if (gc) atomicAdd(gc + (size_t)c * p.C_out + co, (float)sum);
      }
    }
  }
  __syncthreads();
  if (grad_x) {
    float* gxc = grad_x + ((size_t)n * p.C_in + c) * p.H * p.W + (size_t)r0 * p.W;
    for (int i = threadIdx.x; i < (r1 - r0) * p.W; i += blockDim.x) gxc[i] = (float)tile[i];
  }
}

// The same for dilation 1, stride 1 (below) or 2 (two adjacent outputs per thread, 3 x 5 input values, 15 slots) and
// an output width that is a multiple of the outputs per thread.  Planes of at most 1024 outputs (the
// 32 x 32, 16 x 16 and 8 x 8 maps of the paper's CIFAR networks): workgroup = (input channel c, G images whose planes
// together have at most 1024 outputs).  Larger planes: workgroup = (image, input channel, band of RB input rows); it
// scans the RB + 2 output rows whose windows reach the band (at most 1024 outputs) and an output counts for the
// parameter gradients in the band that owns the first row of its window.  A thread owns FOUR ADJACENT output pixels
// of a row of one image.
// Their windows overlap, so the thread keeps 3 x 6 input values instead of 4 x 9, reads gy with one 16-byte load per
// output channel, and -- the point -- adds a winner's gradient into one of 18 fp64 slots of its own in LDS
// ([slot][thread]: no other thread touches them, so a plain read-add-write serves: 8 LDS clocks where the atomic
// into the shared plane costs 13 and, with the winners of neighbouring pixels falling on the same element, 20 on
// average; fp32 slots would halve that again but miss the 1e-5 relative gate at 64 output channels).  After the
// last output channel an input element is the sum of the at most six slots that cover it, read in a fixed order: no
// plane in LDS, no atomics, and grad_x is the same on every run.  The parameter gradients are formed as in the
// kernel above, in chunks of SUMQ_COB output channels.
// Bins of one (output channel, branch, replica): 9 taps, the coefficient sum, one pad (an odd stride spreads the
// replicas over the LDS banks).  With the slots 48 KB of LDS: three workgroups per compute unit.  Measured on the
// 32 x 32, 64 -> 64 layer: 8 channels x 8 replicas 1.27 ms, 4 x 16 1.28, 2 x 8 (four workgroups) 1.28, 8 x 4 1.48,
// 2 x 32 1.46, 16 x 8 (two workgroups) 1.46, 1 x 8 1.38; four slots for the coefficient sum (fewer adds to one
// address) at a stride of 13: 1.32.
constexpr int SUMQ_COB = 8, SUMQ_REP = 8, SUMQ_BS = 11;
constexpr int SUMQ_PRIV_BYTES = 18 * 256 * 8;
template <int MODE, int S>
__global__ __launch_bounds__(256) void sum_bwd_fused3x3_quad_kernel(Params p, const float* __restrict__ x,
                                                                    const float* __restrict__ w_min,
                                                                    const float* __restrict__ w_max,
                                                                    const float* __restrict__ alpha,
                                                                    const float* __restrict__ beta,
                                                                    const float* __restrict__ gy,
                                                                    float* __restrict__ grad_x,
                                                                    float* __restrict__ grad_w_min,
                                                                    float* __restrict__ grad_w_max,
                                                                    float* __restrict__ grad_alpha,
                                                                    float* __restrict__ grad_beta, int COB, int G, int RB,
                                                                    int n_bands) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr bool TWO = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  constexpr int NBR = (DO_MIN && DO_MAX) ? 2 : 1;
  constexpr int REP = SUMQ_REP;
  constexpr int BS = SUMQ_BS;
  constexpr int PXT = 4 / S;               // adjacent outputs of a thread: 4 at stride 1, 2 at stride 2
  constexpr int NQ = S * (PXT - 1) + 3;    // input columns their windows span: 6 / 5
  const int NBINS = COB * NBR * REP * BS;
  extern __shared__ double lds_d[];
  const int band = blockIdx.x % n_bands;
  const int c = (blockIdx.x / n_bands) % p.C_in;
  const int n0 = (blockIdx.x / (n_bands * p.C_in)) * G;  // first image of the group
  // the band owns the input rows [r0, r1); the output rows whose windows reach them are scanned
  const int r0 = band * RB, r1 = min(r0 + RB, p.H);
  const int lo_num = r0 + p.ph - 2;  // first output row whose window (rows S * oh - ph .. + 2) reaches row r0
  const int oh_lo = lo_num <= 0 ? 0 : (lo_num + S - 1) / S, oh_hi = min(p.Ho - 1, (r1 - 1 + p.ph) / S);
  const int srows = max(oh_hi - oh_lo + 1, 0);
  const int xr0 = max(0, S * oh_lo - p.ph), xr1 = srows > 0 ? min(p.H, S * oh_hi - p.ph + 3) : xr0;  // input rows read
  double* const priv = lds_d;                      // [18][256]
  float* const xs = (float*)lds_d;                 // [G][(xr1 - xr0) x W], before the slots are cleared
  double* const bins = lds_d + 18 * 256;           // [COB][NBR][REP][BS]
  const int HW = p.H * p.W;
  const int XW = (xr1 - xr0) * p.W;
  for (int i = threadIdx.x; i < G * XW; i += blockDim.x) {
    const int img = i / XW;
    xs[i] = n0 + img < p.N ? x[((size_t)(n0 + img) * p.C_in + c) * HW + (size_t)xr0 * p.W + (i - img * XW)] : 0.f;
  }
  for (int e = threadIdx.x; e < NBINS; e += blockDim.x) bins[e] = 0.0;
  __syncthreads();
  const size_t plane = (size_t)p.Ho * p.Wo;
  const int qrow = p.Wo / PXT;            // threads per output row
  const int quads = srows * qrow;         // per image
  const int img = quads > 0 ? min((int)threadIdx.x / quads, G - 1) : 0;
  const bool live = (int)threadIdx.x < G * quads && n0 + img < p.N;
  const int lq = live ? (int)threadIdx.x - img * quads : 0;
  const int srow = lq / qrow;
  const int oh = oh_lo + srow, ow0 = PXT * (lq - srow * qrow);
  const int ih0 = S * oh - p.ph, iw0 = S * ow0 - p.pw;
  // an output counts for the parameter gradients in the band that owns the first row of its window inside the image
  const bool own = live && max(ih0, 0) >= r0 && max(ih0, 0) < r1;
  float xw[3][NQ];  // padding = NaN: never an extremum
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      const int ih = ih0 + r, iw = iw0 + q;
      const bool ok = ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
      xw[r][q] = ok ? xs[img * XW + (ih - xr0) * p.W + iw] : __uint_as_float(0x7fc00000u);
    }
  __syncthreads();  // every window is in registers: the slots take the place of the plane
  double* const mine = priv + threadIdx.x;
#pragma unroll
  for (int sl = 0; sl < 3 * NQ; ++sl) mine[sl * 256] = 0.0;
  double* const mybins = bins + (size_t)(threadIdx.x & (REP - 1)) * BS;
  const float* gyq = gy + (size_t)(live ? n0 + img : 0) * p.C_out * plane + (size_t)oh * p.Wo + ow0;
  for (int cob = 0; cob < p.C_out; cob += COB) {
    const int ncb = min(COB, p.C_out - cob);
    if (live) {
      for (int b = 0; b < ncb; ++b) {  // uniform over the workgroup
        const int co = cob + b;
        const float* ka = DO_MIN ? w_min + ((size_t)co * p.C_in + c) * 9 : nullptr;
        const float* kb = DO_MAX ? w_max + ((size_t)co * p.C_in + c) * 9 : nullptr;
        const double ca = TWO ? (double)coef_of(alpha, c, co, p.C_out) : 1.0;
        const double cb = TWO ? (double)coef_of(beta, c, co, p.C_out) : 1.0;
        double* const bn = mybins + (size_t)b * NBR * REP * BS;
        float gk[PXT];
        if constexpr (S == 1) {
          const float4 g4 = *(const float4*)(gyq + (size_t)co * plane);
          gk[0] = g4.x; gk[1] = g4.y; gk[2] = g4.z; gk[3] = g4.w;
        } else {
          const float2 g2 = *(const float2*)(gyq + (size_t)co * plane);
          gk[0] = g2.x; gk[1] = g2.y;
        }
        float s_min = 0.f, s_max = 0.f;  // coefficient sums over the thread's pixels
#pragma unroll
        for (int k = 0; k < PXT; ++k) {
          const double g = (double)gk[k];
          float s1[9], s2[9];
#pragma unroll
          for (int t = 0; t < 9; ++t) {
            if (DO_MIN) s1[t] = __fadd_rn(xw[t / 3][S * k + t % 3], ka[t]);
            if (DO_MAX) s2[t] = (MODE == TCONV_COMPOUND) ? s1[t] : __fadd_rn(xw[t / 3][S * k + t % 3], kb[t]);
          }
          if (DO_MIN) {
            float bmin; int row, col;
            window_extremum9_rc<false>(s1, bmin, row, col);
            const double v = ca * g;
            mine[(row * NQ + col + S * k) * 256] += v;  // slot (row, S * k + column)
            if (own) atomicAdd(bn + (row * 3 + col), v);
            s_min = fmaf(gk[k], bmin, s_min);
          }
          if (DO_MAX) {
            float bmax; int row, col;
            window_extremum9_rc<true>(s2, bmax, row, col);
            const double v = cb * g;
            mine[(row * NQ + col + S * k) * 256] += v;
            if (own) atomicAdd(bn + (NBR - 1) * REP * BS + (row * 3 + col), v);
            s_max = fmaf(gk[k], bmax, s_max);
          }
        }
        if (TWO && own) {
          atomicAdd(bn + 9, (double)s_min);
          atomicAdd(bn + REP * BS + 9, (double)s_max);
        }
      }
    }
    __syncthreads();
    // publish the chunk (replicas in a fixed order, one fp32 atomic per value) and clear what was read
    for (int v = threadIdx.x; v < COB * NBR * 10; v += blockDim.x) {
      const int b = v / (NBR * 10), r = v - b * (NBR * 10), br = r / 10, t = r - br * 10;
      double sum = 0.0;
#pragma unroll
      for (int q = 0; q < REP; ++q) {
        double* const e = bins + ((size_t)(b * NBR + br) * REP + q) * BS + t;
        sum += *e;
        *e = 0.0;
      }
      const bool is_max = DO_MAX && (NBR == 1 || br == 1);
      const int co = cob + b;
      if (b < ncb) {
        if (t < 9) {
          float* gw = is_max ? grad_w_max : grad_w_min;
          if (gw) atomicAdd(gw + ((size_t)co * p.C_in + c) * 9 + t, (float)sum);
        } else if (TWO) {
          float* gc = is_max ? grad_beta : grad_alpha;
          if (gc) atomicAdd(gc + (size_t)c * p.C_out + co, (float)sum);
        }
      }
    }
    __syncthreads();
  }
  // An input element (ih, iw) lies in slot (r, q) of the thread whose outputs start at row (ih + ph - r) / S and column
  // (iw + pw - q) / S; that column is a multiple of PXT, i.e. iw + pw - q a multiple of 4, for one or two q in
  // 0 .. NQ - 1, and at stride 2 the row exists for the r of one parity only.  Slots outside the image never received
  // anything.
  const int BW = (r1 - r0) * p.W;
  for (int i = threadIdx.x; i < G * BW; i += blockDim.x) {
    const int im = i / BW, pos = i - im * BW;
    if (n0 + im >= p.N) break;
    const int br = pos / p.W, iw = pos - br * p.W, ih = r0 + br;
    const int q0 = (iw + p.pw) & 3;
    double sum = 0.0;
#pragma unroll
    for (int r = 0; r < 3; ++r) {
      const int on = ih + p.ph - r;
      if (on < 0 || (S == 2 && (on & 1))) continue;
      const int oh2 = on / S;
      if (oh2 < oh_lo || oh2 > oh_hi) continue;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int q = q0 + 4 * j, oc = (iw + p.pw - q) / S;  // iw + pw - q is a multiple of 4 (or negative: skipped)
        if (q < NQ && iw + p.pw - q >= 0 && oc < p.Wo)
          sum += priv[(r * NQ + q) * 256 + im * quads + (oh2 - oh_lo) * qrow + oc / PXT];
      }
    }
    grad_x[((size_t)(n0 + im) * p.C_in + c) * HW + (size_t)ih * p.W + iw] = (float)sum;
  }
}

__global__ __launch_bounds__(256) void sum_fill_zero_kernel(float* __restrict__ p, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0.f;
}

void zero_fill(float* p, size_t n, hipStream_t s) {  // a kernel, so that the call can sit in a captured graph
  if (!p || n == 0) return;
  size_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(sum_fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, n);
}

bool tiled_ok(const Params& p) {
  if (p.KH != 3 || p.KW != 3 || p.sh != p.sw || p.dh != p.dw) return false;
  const bool geo = (p.sh == 1 && (p.dh == 1 || p.dh == 2)) || (p.sh == 2 && p.dh == 1);
  if (!geo) return false;
  if (p.pw > p.dw || p.Wo < 4) return false;
  if (p.W < 8) return false;  // a row is loaded as a run of 8 (or 4) columns
  if ((size_t)p.N * p.C_in * p.H * p.W * 4 >= 0xfffff000ull) return false;
  return true;
}

template <int MODE, typename TO>
hipError_t launch_fwd(const Params& p, const SumArgs& a, hipStream_t s) {
  const char* e = getenv("TCONV_FORWARD_KERNEL");
  const bool force_generic = e && strcmp(e, "generic") == 0;
  if (tiled_ok(p) && !force_generic) {
    // Small layers (the maps of a CIFAR network) have too few waves at 8 outputs x 4 output channels per lane: fewer
    // outputs (stride 1) or channels per lane then.  1 channel per lane gains nothing more, nor do fewer waves per
    // workgroup at the same number of waves.
    const char* te = getenv("TCONV_SUM_FWD_TN");  // testing aid: 2 or 4 output channels per lane
    const char* pe = getenv("TCONV_SUM_FWD_PX");  // testing aid: 4 or 8 outputs per lane at stride 1
    const int wpb = WAVES;
    auto nwaves = [&](int tn_, int px_) {
      const long long units = (long long)p.N * p.Ho * ((p.Wo + px_ - 1) / px_);
      return ((units + 63) / 64) * (((long long)p.C_out + tn_ - 1) / tn_);
    };
    int tn = 4, px = p.sh == 1 ? 8 : 4;
    if (p.sh == 1) {
      // the first of (4 channels, 8 outputs), (4, 4), (2, 8), (2, 4) per lane that gives two waves per SIMD, else the last.
      // Measured (us, the four forms in that order): [128, 16, 32, 32] -> 16: 33.2 / 28.8 / 34.9 / 35.4,
      // [128, 32, 16, 16] -> 32: 55.5 / 35.6 / 32.3 / 33.0, [128, 64, 8, 8] -> 64: 100.8 / 63.5 / 55.7 / 38.7.
      static const int forms[4][2] = {{4, 8}, {4, 4}, {2, 8}, {2, 4}};
      int pick = 3;
      for (int f = 0; f < 4; ++f)
        if (nwaves(forms[f][0], forms[f][1]) >= 2048) { pick = f; break; }
      tn = forms[pick][0];
      px = forms[pick][1];
    } else if (nwaves(4, px) < 1024) {
      tn = 2;
    }
    if (te && (te[0] == '2' || te[0] == '4') && te[1] == 0) tn = te[0] - '0';
    if (p.sh == 1 && pe && (pe[0] == '4' || pe[0] == '8') && pe[1] == 0) px = pe[0] - '0';
    if (p.Wo < px) px = 4;  // Wo >= 4 here
    const int segs = (p.Wo + px - 1) / px;
    const long long n_units = (long long)p.N * p.Ho * segs;
    const long long ublocks = (n_units + 63) / 64;
    const int n_groups = (p.C_out + tn - 1) / tn;
    const long long blocks = ublocks * ((n_groups + wpb - 1) / wpb);
    if (blocks > 0x7ffffff0LL) return hipErrorInvalidValue;
    // contiguous runs per XCD while the kernels and coefficients are small next to an L2 (as for the full-window kernel)
    const long long w_bytes = (long long)p.C_out * p.K * (long long)sizeof(float) * (MODE == TCONV_PARALLEL ? 2 : 1);
    const char* xe = getenv("TCONV_XCD_RUNS");
    const int xcd_runs = xe ? atoi(xe) : (w_bytes <= 2LL * 1024 * 1024 ? 1 : 0);
    const unsigned grid = (unsigned)(((blocks + 7) / 8) * 8);
    const TO* x = (const TO*)a.x;
    TO* y = (TO*)a.y;
#define TCONV_SUM_FWD(D_, S_, TN_, PX_)                                                                                     \
  hipLaunchKernelGGL((sum_fwd_tiled3x3_kernel<MODE, D_, S_, TO, TN_, PX_>), dim3(grid), dim3(wpb * 64), 0, s, p, x, a.w_min, \
                     a.w_max, a.alpha, a.beta, y, segs, (int)n_units, n_groups, (int)blocks, xcd_runs, wpb)
#define TCONV_SUM_FWD_TN(D_, S_, PX_) \
  do { if (tn == 4) TCONV_SUM_FWD(D_, S_, 4, PX_); else TCONV_SUM_FWD(D_, S_, 2, PX_); } while (0)
    if (p.sh == 2) TCONV_SUM_FWD_TN(1, 2, 4);
    else if (p.dh == 1) { if (px == 8) TCONV_SUM_FWD_TN(1, 1, 8); else TCONV_SUM_FWD_TN(1, 1, 4); }
    else { if (px == 8) TCONV_SUM_FWD_TN(2, 1, 8); else TCONV_SUM_FWD_TN(2, 1, 4); }
#undef TCONV_SUM_FWD_TN
#undef TCONV_SUM_FWD
  } else if (sizeof(TO) != 4) {
    return hipErrorInvalidValue;  // bf16 storage: the tiled kernel only
  } else {
    const size_t total = (size_t)p.N * p.C_out * p.Ho * p.Wo;
    hipLaunchKernelGGL(sum_fwd_generic_kernel<MODE>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, p,
                       a.x, a.w_min, a.w_max, a.alpha, a.beta, a.y);
  }
  return hipGetLastError();
}

template <int MODE>
hipError_t launch_bwd(const Params& p, const SumArgs& a, const SumGrads& g, hipStream_t s) {
  const int KK = p.KH * p.KW;
  {
    // 3x3 windows with the input gradient AND parameter gradients wanted: one kernel, one winner search
    float* fmin = g.grad_w_min;
    float* fmax = g.grad_w_max;
    if (MODE == TCONV_COMPOUND) fmin = fmax = (g.grad_w_min ? g.grad_w_min : g.grad_w_max);
    const bool want_par = (MODE != TCONV_MAX && fmin) || (MODE != TCONV_MIN && fmax) || g.grad_alpha || g.grad_beta;
    const char* sep = getenv("TCONV_SUM_BWD");  // testing aid: "separate" keeps the two-kernel path
    if (p.KH == 3 && p.KW == 3 && g.grad_x && want_par && !(sep && strcmp(sep, "separate") == 0)) {
      constexpr int NBR = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL) ? 2 : 1;
      int COB = p.C_out < 16 ? p.C_out : 16;  // 16 channels x 16 replicas x 2 branches x 11 doubles = 45 KB
      const size_t bins_bytes = (size_t)SUMF_REP * COB * NBR * 11 * 8;
      const size_t budget = 60 * 1024;
      const int eh = p.dh * 2;
      int TH = p.H;
      auto bytes = [&](int th) {
        const long long xrows = (long long)th + 2LL * eh + p.sh;
        return (size_t)th * p.W * 8 + bins_bytes + (size_t)(xrows < p.H ? xrows : p.H) * p.W * 4;
      };
      while (TH > 1 && bytes(TH) > budget) TH = (TH + 1) / 2;
      const int n_bands = (p.H + TH - 1) / TH;
      const long long blocks = (long long)p.N * p.C_in * n_bands;
      if (bytes(TH) <= 64 * 1024 && blocks <= 0x7fffffffLL) {
        const size_t nw = (size_t)p.C_out * p.C_in * KK, nab = (size_t)p.C_in * p.C_out;
        if (MODE != TCONV_MAX) zero_fill(fmin, nw, s);
        if (MODE == TCONV_MAX || MODE == TCONV_PARALLEL) zero_fill(fmax, nw, s);
        zero_fill(g.grad_alpha, nab, s);
        zero_fill(g.grad_beta, nab, s);
        // stride 1, dilation 1, rows of a multiple of 4 outputs, gy readable in 16-byte pieces: a thread owns four
        // adjacent outputs and its own gradient slots.  Planes of at most 1024 outputs: one band, as many images to a
        // workgroup as fill its threads.  Larger planes: one image, bands of RB input rows whose RB + 2 scanned
        // output rows fill the threads (at least 4 rows to a band: at most 1.5 x the outputs are scanned).
        const long long plane = (long long)p.Ho * p.Wo;
        const int S = p.sh, pxt = S == 2 ? 2 : 4;  // adjacent outputs of a thread
        const int qrow = p.Wo / pxt;
        int G = 0, RB = p.H, nb = 1;
        if (plane > 0 && plane <= 256 * pxt) {
          G = (int)std::min<long long>(256 * pxt / plane, p.N);
          if (G * plane <= 128 * pxt) G = 0;  // too few outputs for the threads
        } else if (qrow >= 1 && qrow <= 42) {
          G = 1;
          RB = S * (256 / qrow - 2);
          nb = (p.H + RB - 1) / RB;
        }
        const long long xrows = std::min<long long>((long long)RB + 6, p.H);  // input rows a band's scanned outputs read, at most
        const bool quad = p.sh == p.sw && (S == 1 || S == 2) && p.dh == 1 && p.dw == 1 && p.Wo % pxt == 0 && G >= 1 &&
                          (size_t)G * xrows * p.W * 4 <= (size_t)SUMQ_PRIV_BYTES &&
                          (long long)((p.N + G - 1) / G) * p.C_in * nb <= 0x7fffffffLL &&
                          ((uintptr_t)g.gy & 15) == 0 && !(sep && strcmp(sep, "spread") == 0);
        if (quad) {
          const int cobq = SUMQ_COB;
          const size_t qbytes = (size_t)SUMQ_PRIV_BYTES + (size_t)SUMQ_REP * cobq * NBR * SUMQ_BS * 8;
          const long long groups = ((long long)p.N + G - 1) / G;
          const dim3 qgrid((unsigned)(groups * p.C_in * nb));
          if (S == 1)
            hipLaunchKernelGGL((sum_bwd_fused3x3_quad_kernel<MODE, 1>), qgrid, dim3(256), qbytes, s, p, a.x, a.w_min,
                               a.w_max, a.alpha, a.beta, g.gy, g.grad_x, fmin, fmax, g.grad_alpha, g.grad_beta, cobq, G,
                               RB, nb);
          else
            hipLaunchKernelGGL((sum_bwd_fused3x3_quad_kernel<MODE, 2>), qgrid, dim3(256), qbytes, s, p, a.x, a.w_min,
                               a.w_max, a.alpha, a.beta, g.gy, g.grad_x, fmin, fmax, g.grad_alpha, g.grad_beta, cobq, G,
                               RB, nb);
          return hipGetLastError();
        }
        if (n_bands == 1)
          hipLaunchKernelGGL((sum_bwd_fused3x3_kernel<MODE, true>), dim3((unsigned)blocks), dim3(256), bytes(TH), s, p,
                             a.x, a.w_min, a.w_max, a.alpha, a.beta, g.gy, g.grad_x, fmin, fmax, g.grad_alpha,
                             g.grad_beta, TH, n_bands, COB);
        else
          hipLaunchKernelGGL((sum_bwd_fused3x3_kernel<MODE, false>), dim3((unsigned)blocks), dim3(256), bytes(TH), s, p,
                             a.x, a.w_min, a.w_max, a.alpha, a.beta, g.gy, g.grad_x, fmin, fmax, g.grad_alpha,
                             g.grad_beta, TH, n_bands, COB);
        return hipGetLastError();
      }
    }
  }
  if (g.grad_x) {
    // band of input rows per workgroup: fp64 sums (8 B) plus the fp32 input rows its windows read
    const size_t budget = 60 * 1024;
    const int eh = p.dh * (p.KH - 1);
    int TH = p.H;
    auto bytes = [&](int th) {
      const long long xrows = (long long)th + 2LL * eh + p.sh;  // upper bound of the rows read
      return (size_t)th * p.W * 8 + (size_t)(xrows < p.H ? xrows : p.H) * p.W * 4;
    };
    while (TH > 1 && bytes(TH) > budget) TH = (TH + 1) / 2;
    if (bytes(TH) > 64 * 1024) return hipErrorInvalidValue;  // rows too long for this kernel
    const int n_bands = (p.H + TH - 1) / TH;
    const long long blocks = (long long)p.N * p.C_in * n_bands;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (p.KH == 3 && p.KW == 3)
      hipLaunchKernelGGL(sum_bwd_x3x3_kernel<MODE>, dim3((unsigned)blocks), dim3(256), bytes(TH), s, p, a.x,
                         a.w_min, a.w_max, a.alpha, a.beta, g.gy, g.grad_x, TH, n_bands);
    else
      hipLaunchKernelGGL(sum_bwd_x_kernel<MODE>, dim3((unsigned)blocks), dim3(256), bytes(TH), s, p, a.x, a.w_min,
                         a.w_max, a.alpha, a.beta, g.gy, g.grad_x, TH, n_bands);
  }
  float* gmin = g.grad_w_min;
  float* gmax = g.grad_w_max;
  if (MODE == TCONV_COMPOUND) gmin = gmax = (g.grad_w_min ? g.grad_w_min : g.grad_w_max);
  const bool want_w = (MODE != TCONV_MAX && gmin) || (MODE != TCONV_MIN && gmax) || g.grad_alpha || g.grad_beta;
  if (want_w) {
    const size_t nw = (size_t)p.C_out * p.C_in * KK, nab = (size_t)p.C_in * p.C_out;
    if (MODE != TCONV_MAX) zero_fill(gmin, nw, s);
    if (MODE == TCONV_MAX || MODE == TCONV_PARALLEL) zero_fill(gmax, nw, s);
    zero_fill(g.grad_alpha, nab, s);
    zero_fill(g.grad_beta, nab, s);
    const long long pairs = (long long)p.C_out * p.C_in;
    if (pairs > 0x7fffffffLL) return hipErrorInvalidValue;
    int slices = (int)((1024 + pairs - 1) / pairs);  // enough workgroups to fill the chip
    if (slices > p.N) slices = p.N;
    if (slices > 65535) slices = 65535;
    const int n_per_block = (p.N + slices - 1) / slices;
    const dim3 grid((unsigned)pairs, (unsigned)((p.N + n_per_block - 1) / n_per_block));
    constexpr int NBR = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL) ? 2 : 1;
    int nt = 256;  // threads (a power of two): fewer for large kernel windows, whose sums fill the LDS
    while (nt > 64 && (size_t)NBR * (KK + 1) * nt * sizeof(double) > 64 * 1024) nt /= 2;
    const size_t lds = (size_t)NBR * (KK + 1) * nt * sizeof(double);
    if (lds > 64 * 1024) return hipErrorInvalidValue;  // kernel window too large for this kernel
    if (p.KH == 3 && p.KW == 3 && (size_t)p.N * p.C_in * p.H * p.W * 4 < 0xfffff000ull) {  // 32-bit byte offsets into x
      const long long n_coblocks = (p.C_out + SUMW_CB - 1) / SUMW_CB, wgs = n_coblocks * p.C_in;
      int sl = (int)((2048 + wgs - 1) / wgs);  // enough workgroups to fill the chip several times over
      if (sl > p.N) sl = p.N;
      if (sl > 65535) sl = 65535;
      const int npb = (p.N + sl - 1) / sl;
      if (wgs > 0x7fffffffLL) return hipErrorInvalidValue;
      hipLaunchKernelGGL(sum_bwd_w3x3_blk_kernel<MODE>, dim3((unsigned)wgs, (unsigned)((p.N + npb - 1) / npb)), dim3(256),
                         0, s, p, a.x, a.w_min, a.w_max, a.alpha, a.beta, g.gy, gmin, gmax, g.grad_alpha, g.grad_beta,
                         npb, (int)n_coblocks);
    }
    else
      hipLaunchKernelGGL(sum_bwd_w_kernel<MODE>, grid, dim3(nt), lds, s, p, a.x, a.w_min, a.w_max, a.alpha, a.beta,
                       g.gy, gmin, gmax, g.grad_alpha, g.grad_beta, n_per_block);
  }
  return hipGetLastError();
}

}  // namespace

namespace {

__global__ __launch_bounds__(256) void sum_widen_kernel(const bf16_t* __restrict__ src, float* __restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    dst[i] = __uint_as_float((unsigned)src[i] << 16);
}

void widen(const void* src, float* dst, size_t n, hipStream_t s) {
  size_t blocks = (n + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(sum_widen_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const bf16_t*)src, dst, n);
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

// bf16 storage: fp32 copies of the kernel tensors (they are read as scalars, in whole dwords) and, for the backward
// pass, of x; returns the copies' pointers in a
void widen_operands(const Params& p, SumArgs& a, bool with_x, void* workspace, hipStream_t s) {
  char* ws = (char*)workspace;
  const size_t nw = (size_t)p.C_out * p.K;
  const bool use_min = p.mode != TCONV_MAX, use_max = p.mode != TCONV_MIN;
  const bool shared = p.mode == TCONV_COMPOUND;  // one kernel tensor behind both pointers
  const float* wmin_f = nullptr;
  if (use_min) {
    widen(a.w_min, (float*)ws, nw, s);
    wmin_f = (const float*)ws;
    ws += align256(nw * 4);
  }
  const float* wmax_f = wmin_f;
  if (use_max && !shared) {
    widen(a.w_max, (float*)ws, nw, s);
    wmax_f = (const float*)ws;
    ws += align256(nw * 4);
  }
  a.w_min = use_min ? wmin_f : nullptr;
  a.w_max = use_max ? wmax_f : nullptr;
  if (with_x) {
    const size_t nx = (size_t)p.N * p.C_in * p.H * p.W;
    widen(a.x, (float*)ws, nx, s);
    a.x = (const float*)ws;
  }
}

}  // namespace

size_t sum_workspace(const Params& p, int dtype, bool backward) {
  if (dtype != TCONV_BF16) return 0;
  const size_t nw = (size_t)p.C_out * p.K;
  size_t b = align256(nw * 4) * (p.mode == TCONV_PARALLEL ? 2 : 1);
  if (backward) b += align256((size_t)p.N * p.C_in * p.H * p.W * 4);
  return b;
}

bool sum_forward_supported(const Params& p, int dtype) {
  if (dtype == TCONV_F32) return true;
  const char* e = getenv("TCONV_FORWARD_KERNEL");
  return dtype == TCONV_BF16 && tiled_ok(p) && !(e && strcmp(e, "generic") == 0);
}

template <typename TO>
static hipError_t launch_sum_forward_t(const Params& p, const SumArgs& a, hipStream_t s) {
  switch (p.mode) {
    case TCONV_MAX: return launch_fwd<TCONV_MAX, TO>(p, a, s);
    case TCONV_MIN: return launch_fwd<TCONV_MIN, TO>(p, a, s);
    case TCONV_COMPOUND: return launch_fwd<TCONV_COMPOUND, TO>(p, a, s);
    default: return launch_fwd<TCONV_PARALLEL, TO>(p, a, s);
  }
}

// bf16 storage (x, kernels, y; workspace of sum_workspace bytes): x is read as bf16 by the kernel, y rounded on store
hipError_t launch_sum_forward(const Params& p, int dtype, const SumArgs& a0, void* workspace, hipStream_t s) {
  if (dtype != TCONV_BF16) return launch_sum_forward_t<float>(p, a0, s);
  SumArgs a = a0;
  widen_operands(p, a, false, workspace, s);
  return launch_sum_forward_t<bf16_t>(p, a, s);
}

// bf16 storage of x and the kernels: the gradient kernels run on fp32 copies (the layer is bound by arithmetic, the
// copies are a few per cent of its traffic)
hipError_t launch_sum_backward(const Params& p, int dtype, const SumArgs& a0, const SumGrads& g, void* workspace,
                               hipStream_t s) {
  SumArgs a = a0;
  if (dtype == TCONV_BF16) widen_operands(p, a, true, workspace, s);
  switch (p.mode) {
    case TCONV_MAX: return launch_bwd<TCONV_MAX>(p, a, g, s);
    case TCONV_MIN: return launch_bwd<TCONV_MIN>(p, a, g, s);
    case TCONV_COMPOUND: return launch_bwd<TCONV_COMPOUND>(p, a, g, s);
    default: return launch_bwd<TCONV_PARALLEL>(p, a, g, s);
  }
}

const char* sum_forward_kernel_name(const Params& p) {
  const char* e = getenv("TCONV_FORWARD_KERNEL");
  return (tiled_ok(p) && !(e && strcmp(e, "generic") == 0)) ? "sum_tiled3x3" : "sum_generic";
}

}  // namespace tconv
