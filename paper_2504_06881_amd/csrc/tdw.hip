// Depthwise tropical convolution layers on gfx950: forward and backward.
//
// Layer: every output channel co reads ONE input channel c = co / mult (mult = C_out / C_in), so the
// layer is the base operator of paper Sec. 3.1 applied per channel,
//   m = min over the window of x + w_min[co],  M = max over the window of x + w_max[co],
//   y = M | m | alpha[co]*m + beta[co]*M  (Sec. 3.5 / 3.6 combination; used in place of the depthwise
//   convolutions of the MobileNetV2 variants, Sec. 5).
// With 9 candidates per output and 8-9 bytes of traffic per output the layer sits on the HBM side of the
// roofline (20 vector instructions of arithmetic per output against 8 bytes), so the kernels are built around
// bytes; what they measure at is about half the HBM rate, because finding the two winning taps exactly costs
// 18 more instructions per output and branch than the arithmetic itself:
//   * forward writes, next to y, ONE byte per output that packs both winning taps (low nibble: min-plus
//     tap, high nibble: max-plus tap); backward reads gy and that byte instead of re-deriving the winners
//     from x (4 more bytes per output and several times the arithmetic);
//   * forward, 3x3: a wave stages the input tile of 64 x 4 outputs in its own slice of LDS (padding as NaN,
//     which v_min3 / v_max3 ignore), each lane then owns 4 consecutive outputs of one row; no workgroup
//     barrier anywhere;
//   * backward w.r.t. the input is a GATHER: the lane that owns an input pixel visits the 9 outputs whose
//     window covers it and adds the gradient of those that picked it.  No atomics, no zero fill, a fixed
//     summation order;
//   * the kernel / coefficient gradients are per-channel reductions: per-thread partial sums in LDS, one
//     float atomic per workgroup and result element.
#include <stdlib.h>
#include <string.h>

#include "tile_common.h"
// after tile_common.h: the blocks header relies on the HIP runtime declarations included there
#include <tile_blocks_gfx950.h>

namespace tconv {
namespace {

using namespace tile;

__device__ __forceinline__ float quiet_nan() { return __uint_as_float(0x7fc00000u); }

typedef float f4a __attribute__((ext_vector_type(4)));  // 16-byte aligned
typedef int i4a __attribute__((ext_vector_type(4)));
typedef unsigned u1a __attribute__((aligned(1)));       // 4 winner bytes at any address

// N consecutive floats from LDS at any 4-byte aligned address (gfx950 reads unaligned vectors from LDS)
template <int N>
__device__ __forceinline__ void lds_run(float* dst, const float* src) {
  if constexpr (N >= 4) {
    const f4u v = *(const f4u*)src;
    dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    lds_run<N - 4>(dst + 4, src + 4);
  } else if constexpr (N >= 2) {
    const f2u v = *(const f2u*)src;
    dst[0] = v.x; dst[1] = v.y;
    lds_run<N - 2>(dst + 2, src + 2);
  } else if constexpr (N == 1) {
    dst[0] = src[0];
  }
}

// sum over the 64 lanes of a wave, returned in every lane
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
  return v;
}

// y of one output from its branch extrema
template <int MODE>
__device__ __forceinline__ float dw_combine(float m, float M, float a, float b) {
  if (MODE == TCONV_MAX) return M;
  if (MODE == TCONV_MIN) return m;
  return combine(a, m, b, M);
}

// Extremum of the 9 sums of a window and (if wanted) its lowest tap: one v_min3 / v_max3 per row, one over the row
// results, then the first row and the first column of it that equal the extremum - 13 instructions for the tap
// where a compare-and-select per tap takes 18.  NaN sums (padding) are ignored and equal nothing.
template <bool WANT_MAX, bool WANT_TAP>
__device__ __forceinline__ void dw_extremum9(const float (&s)[9], float& best, int& tap) {
  float r[3];
#pragma unroll
  for (int i = 0; i < 3; ++i)
    r[i] = WANT_MAX ? fmaxf(fmaxf(s[3 * i], s[3 * i + 1]), s[3 * i + 2]) : fminf(fminf(s[3 * i], s[3 * i + 1]), s[3 * i + 2]);
  best = WANT_MAX ? fmaxf(fmaxf(r[0], r[1]), r[2]) : fminf(fminf(r[0], r[1]), r[2]);
  if (WANT_TAP) {
    const bool c0 = r[0] == best, c1 = r[1] == best;
    const int row = c0 ? 0 : (c1 ? 1 : 2);
    const float a0 = c0 ? s[0] : (c1 ? s[3] : s[6]);
    const float a1 = c0 ? s[1] : (c1 ? s[4] : s[7]);
    const int col = (a0 == best) ? 0 : ((a1 == best) ? 1 : 2);
    tap = row * 3 + col;
  }
}

// 4 consecutive outputs of one row from the 3 x (3*S + 3) input values under them (padding = NaN, which
// v_min3 / v_max3 ignore and which never equals an extremum): y, and the packed winners if wanted.
template <int MODE, int S, bool WANT_IDX>
__device__ __forceinline__ void dw_px4(const float (&xs)[3][3 * S + 3], const float (&wa)[9], const float (&wb)[9],
                                       float a, float b, float (&out)[4], int (&code)[4]) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    float sa[9], sb[9];
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        const float xv = xs[i][q * S + j];
        if (DO_MIN) sa[i * 3 + j] = __fadd_rn(xv, wa[i * 3 + j]);
        if (DO_MAX) sb[i * 3 + j] = (MODE == TCONV_COMPOUND) ? sa[i * 3 + j] : __fadd_rn(xv, wb[i * 3 + j]);
      }
    float m = 0.f, M = 0.f;
    int tm = 0, tM = 0;
    if (DO_MIN) dw_extremum9<false, WANT_IDX>(sa, m, tm);
    if (DO_MAX) dw_extremum9<true, WANT_IDX>(sb, M, tM);
    out[q] = dw_combine<MODE>(m, M, a, b);
    code[q] = tm | (tM << 4);
  }
}

// outputs q >= first_q of a lane's 4 go to y[ob + q] (and their winner bytes to idx[ob + q])
template <bool WANT_IDX>
__device__ __forceinline__ void dw_store4(float* __restrict__ y, uint8_t* __restrict__ idx, size_t ob,
                                          const float (&out)[4], const int (&code)[4], int first_q) {
  store_row<4>(y + ob, out, first_q);
  if (WANT_IDX) {
    if (first_q == 0 && ((uintptr_t)(idx + ob) & 3) == 0) {
      *(unsigned*)(idx + ob) = (unsigned)code[0] | ((unsigned)code[1] << 8) | ((unsigned)code[2] << 16) |
                               ((unsigned)code[3] << 24);
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (q >= first_q) idx[ob + q] = (uint8_t)code[q];
    }
  }
}

// The gradient that reaches each of 4 consecutive input pixels through either branch, unscaled: g6 / c6 hold gy
// and the winner bytes of the outputs of rows ih + ph - i (i = 0, 1, 2), columns iw0 + pw - 2 .. + 3.
template <int MODE>
__device__ __forceinline__ void dw_gather4(const float (&g6)[3][6], const int (&c6)[3][6], float (&am)[4],
                                           float (&aM)[4]) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    int cmn[6], cmx[6];
#pragma unroll
    for (int k = 0; k < 6; ++k) { cmn[k] = c6[i][k] & 15; cmx[k] = c6[i][k] >> 4; }
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const int t = i * 3 + j;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (DO_MIN) am[q] += (cmn[q + 2 - j] == t) ? g6[i][q + 2 - j] : 0.f;
        if (DO_MAX) aM[q] += (cmx[q + 2 - j] == t) ? g6[i][q + 2 - j] : 0.f;
      }
    }
  }
}

// quotient of u by d through the multiply-high with inv = floor(2^32 / d) + 1 (inv = 0 stands for d = 1);
// exact while u * d < 2^32
__device__ __forceinline__ unsigned fast_div(unsigned u, unsigned inv) { return inv ? __umulhi(u, inv) : u; }

// ------------------------------------------------------------------------------------------ forward, generic

// One thread per output, any window size, stride, padding, dilation.  Padded taps are skipped; strict
// compares in ascending tap order keep the lowest winning tap.
template <int MODE>
__global__ __launch_bounds__(256) void dw_fwd_generic_kernel(Params p, int mult, const float* __restrict__ x,
                                                             const float* __restrict__ w_min,
                                                             const float* __restrict__ w_max,
                                                             const float* __restrict__ alpha,
                                                             const float* __restrict__ beta, float* __restrict__ y,
                                                             uint8_t* __restrict__ idx) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  const size_t total = (size_t)p.N * p.C_out * p.Ho * p.Wo;
  const size_t o = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= total) return;
  const int ow = (int)(o % p.Wo);
  const int oh = (int)((o / p.Wo) % p.Ho);
  const int co = (int)((o / ((size_t)p.Wo * p.Ho)) % p.C_out);
  const int n = (int)(o / ((size_t)p.Wo * p.Ho * p.C_out));
  const int KK = p.KH * p.KW;
  const float* xp = x + ((size_t)n * p.C_in + co / mult) * p.H * p.W;
  const float* wa = DO_MIN ? w_min + (size_t)co * KK : nullptr;
  const float* wb = DO_MAX ? w_max + (size_t)co * KK : nullptr;
  float m = INFINITY, M = -INFINITY;
  int tm = 0, tM = 0;
  for (int i = 0; i < p.KH; ++i) {
    const int ih = oh * p.sh - p.ph + i * p.dh;
    if (ih < 0 || ih >= p.H) continue;
    for (int j = 0; j < p.KW; ++j) {
      const int iw = ow * p.sw - p.pw + j * p.dw;
      if (iw < 0 || iw >= p.W) continue;
      const float xv = xp[(size_t)ih * p.W + iw];
      const int t = i * p.KW + j;
      if (DO_MIN) {
        const float s = __fadd_rn(xv, wa[t]);
        if (s < m) { m = s; tm = t; }
      }
      if (DO_MAX) {
        const float s = __fadd_rn(xv, wb[t]);
        if (s > M) { M = s; tM = t; }
      }
    }
  }
  float a = 1.f, b = 1.f;
  if (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL) {
    if (alpha) a = alpha[co];
    if (beta) b = beta[co];
  }
  y[o] = dw_combine<MODE>(m, M, a, b);
  if (idx) idx[o] = (uint8_t)(tm | (tM << 4));
}

// ------------------------------------------------------------------------------------------ forward, 3x3 tiled

// A wave owns TH x TW outputs of one (image, output channel) plane: LR = TW/4 lanes side by side, each with
// 4 consecutive outputs of a row, TH = 64 / LR rows.  The last tile of a row is moved left so that it ends
// with the row (its lanes store only the columns the unmoved tile would own), and the last 4-pixel segment
// of a short row likewise.
template <int MODE, int S, int TW, bool WANT_IDX>
__global__ __launch_bounds__(WAVES * 64) void dw_fwd_tiled_kernel(Params p, int mult, const float* __restrict__ x,
                                                                  const float* __restrict__ w_min,
                                                                  const float* __restrict__ w_max,
                                                                  const float* __restrict__ alpha,
                                                                  const float* __restrict__ beta,
                                                                  float* __restrict__ y, uint8_t* __restrict__ idx,
                                                                  int tiles_h, unsigned inv_tiles_h) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr int LR = TW / 4, TH = 64 / LR;
  constexpr int ROWS = (TH - 1) * S + 3, COLS = (TW - 1) * S + 3;
  constexpr int CPR = (COLS + 3 + 3) / 4, PITCH = 4 * CPR;  // 4-float chunks per tile row (any alignment of its start)
  constexpr int NC = 3 * S + 3;                             // input columns under a lane's 4 outputs
  __shared__ __attribute__((aligned(16))) float tile_all[WAVES][ROWS * PITCH];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  // grid: x = tile column, y = groups of WAVES (output channel, tile row) pairs, z = image; the one split that
  // is needed is a multiply-high (an integer division would run on the vector ALU even though it is uniform)
  const int tw = blockIdx.x;
  const unsigned u = blockIdx.y * WAVES + wave;
  const int co = (int)((tiles_h == 1) ? u : __umulhi(u, inv_tiles_h));
  const int th = (int)u - co * tiles_h;
  if (co >= p.C_out) return;  // whole wave; the kernel has no workgroup barrier
  const int n = blockIdx.z;
  const int plane = n * p.C_out + co;
  const int own_w = tw * TW;
  const int org_w = min(own_w, max(p.Wo - TW, 0));
  const int oh0 = th * TH;
  const float* xp = x + ((size_t)n * p.C_in + co / mult) * p.H * p.W;
  const int ih_base = oh0 * S - p.ph, iw_base = org_w * S - p.pw;
  float* const t = tile_all[wave];
  // The tile is fetched in 4-float chunks that start at multiples of 4 in plane columns (tile column 0 is
  // plane column cbase), so a chunk is left of the plane, right of it, inside it, or hangs over the row end
  // by the same dd = (4 - W % 4) % 4 columns everywhere; that last kind is loaded from W - 4 and shifted.
  // All loads are issued before any is consumed: one memory latency per tile.
  const int cbase = (iw_base < 0) ? -4 : (iw_base & ~3);
  const int dd = (4 - (p.W & 3)) & 3;
  constexpr int NCH = ROWS * CPR, NIT = (NCH + 63) / 64;
  f4u stage[NIT];
#pragma unroll
  for (int k = 0; k < NIT; ++k) {
    const int e = min(lane + 64 * k, NCH - 1);
    const int r = e / CPR, q = e - r * CPR;
    const int ih = min(max(ih_base + r, 0), p.H - 1);
    const int start = min(max(cbase + 4 * q, 0), p.W - 4);
    stage[k] = *(const f4u*)(xp + (size_t)ih * p.W + start);
  }
#pragma unroll
  for (int k = 0; k < NIT; ++k) {
    const int e = lane + 64 * k;
    const int r = e / CPR, q = e - r * CPR;
    const int ih = ih_base + r, c0 = cbase + 4 * q;
    const bool row_ok = (ih >= 0 && ih < p.H);
    f4u v = stage[k];
    if (dd != 0 && c0 + 4 > p.W) {  // hangs over the row end (or lies beyond it: then nothing of it is kept)
      const f4u u = v;
      if (dd == 1) { v.x = u.y; v.y = u.z; v.z = u.w; }
      else if (dd == 2) { v.x = u.z; v.y = u.w; }
      else { v.x = u.w; }
    }
    f4a o;
    o.x = (row_ok && c0 >= 0 && c0 < p.W) ? v.x : quiet_nan();
    o.y = (row_ok && c0 >= 0 && c0 + 1 < p.W) ? v.y : quiet_nan();
    o.z = (row_ok && c0 >= 0 && c0 + 2 < p.W) ? v.z : quiet_nan();
    o.w = (row_ok && c0 >= 0 && c0 + 3 < p.W) ? v.w : quiet_nan();
    if (e < NCH) *(f4a*)&t[r * PITCH + 4 * q] = o;
  }
  wave_lds_fence();

  const int r = lane / LR, seg = lane % LR;
  const int oh = oh0 + r;
  const int nominal = org_w + 4 * seg;
  const int lo = max(own_w, nominal);       // first column this lane is responsible for
  const int ow0 = min(nominal, p.Wo - 4);   // first column it computes
  const int first_q = lo - ow0;             // >= 4: nothing to store
  const bool act = (oh < p.Ho) && (first_q < 4);
  const int lc = ow0 * S - p.pw - cbase;  // tile column of the first input column under this lane

  float xs[3][NC];
#pragma unroll
  for (int i = 0; i < 3; ++i) lds_run<NC>(xs[i], &t[(r * S + i) * PITCH + lc]);

  float wa[9], wb[9];
#pragma unroll
  for (int k = 0; k < 9; ++k) {
    wa[k] = DO_MIN ? w_min[(size_t)co * 9 + k] : 0.f;
    wb[k] = DO_MAX ? w_max[(size_t)co * 9 + k] : 0.f;
  }
  float a = 1.f, b = 1.f;
  if (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL) {
    if (alpha) a = alpha[co];
    if (beta) b = beta[co];
  }
  float out[4];
  int code[4];
  dw_px4<MODE, S, WANT_IDX>(xs, wa, wb, a, b, out, code);
  if (!act) return;
  dw_store4<WANT_IDX>(y, idx, ((size_t)plane * p.Ho + oh) * p.Wo + ow0, out, code, first_q);
}

// ------------------------------------------------------------------------------------------ 3x3 by rows (small planes)

// One lane = 4 consecutive outputs (forward) or input pixels (backward) of one row of one plane, with the rows
// of ALL planes numbered consecutively, so that planes much smaller than a wave's tile still fill the wave.
// No LDS: a lane reads the values under its 4 pixels itself (clamped addresses, padding selected afterwards);
// neighbouring lanes touch the same cache lines.  One input channel per output channel (mult == 1), so an
// output plane and its input plane have the same number.
template <int MODE, int S, bool WANT_IDX>
__global__ __launch_bounds__(256) void dw_fwd_rows_kernel(Params p, const float* __restrict__ x,
                                                          const float* __restrict__ w_min,
                                                          const float* __restrict__ w_max,
                                                          const float* __restrict__ alpha,
                                                          const float* __restrict__ beta, float* __restrict__ y,
                                                          uint8_t* __restrict__ idx, int segs, unsigned n_units,
                                                          unsigned inv_segs, unsigned inv_rows, unsigned inv_c) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr int NC = 3 * S + 3;
  const unsigned u = blockIdx.x * 256u + threadIdx.x;
  if (u >= n_units) return;
  const unsigned t = fast_div(u, inv_segs);
  const int seg = (int)(u - t * (unsigned)segs);
  const unsigned plane = fast_div(t, inv_rows);
  const int oh = (int)(t - plane * (unsigned)p.Ho);
  const int co = (int)(plane - fast_div(plane, inv_c) * (unsigned)p.C_out);
  const int ow0 = min(seg * 4, p.Wo - 4);
  const int first_q = seg * 4 - ow0;
  const float* xp = x + (size_t)plane * p.H * p.W;
  float xs[3][NC];
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int ih = oh * S - p.ph + i;
    const bool row_ok = (ih >= 0 && ih < p.H);
    const float* xr = xp + (size_t)min(max(ih, 0), p.H - 1) * p.W;
#pragma unroll
    for (int k = 0; k < NC; ++k) {
      const int iw = ow0 * S - p.pw + k;
      const float v = xr[min(max(iw, 0), p.W - 1)];
      xs[i][k] = (row_ok && iw >= 0 && iw < p.W) ? v : quiet_nan();
    }
  }
  float wa[9], wb[9];
#pragma unroll
  for (int k = 0; k < 9; ++k) {
    wa[k] = DO_MIN ? w_min[(size_t)co * 9 + k] : 0.f;
    wb[k] = DO_MAX ? w_max[(size_t)co * 9 + k] : 0.f;
  }
  float a = 1.f, b = 1.f;
  if (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL) {
    if (alpha) a = alpha[co];
    if (beta) b = beta[co];
  }
  float out[4];
  int code[4];
  dw_px4<MODE, S, WANT_IDX>(xs, wa, wb, a, b, out, code);
  dw_store4<WANT_IDX>(y, idx, ((size_t)plane * p.Ho + oh) * p.Wo + ow0, out, code, first_q);
}

// Dilation 1, stride S = 1 or 2.  At stride 2 an input pixel is read through tap (i, j) only where ih + ph - i and
// iw + pw - j are even: per kernel row at most 4 outputs lie under a lane's 4 pixels, and which (pixel, tap)
// pairs meet which of them depends on the parity of iw0 + pw alone.
template <int MODE, int S, int PAR = -1>
__global__ __launch_bounds__(256) void dw_bwd_x_rows_kernel(Params p, const float* __restrict__ gy,
                                                            const uint8_t* __restrict__ idx,
                                                            const float* __restrict__ alpha,
                                                            const float* __restrict__ beta,
                                                            float* __restrict__ grad_x, int segs, unsigned n_units,
                                                            unsigned inv_segs, unsigned inv_rows, unsigned inv_c) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr bool TWO = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  const unsigned u = blockIdx.x * 256u + threadIdx.x;
  if (u >= n_units) return;
  const unsigned t = fast_div(u, inv_segs);
  const int seg = (int)(u - t * (unsigned)segs);
  const unsigned plane = fast_div(t, inv_rows);
  const int ih = (int)(t - plane * (unsigned)p.H);
  const int c = (int)(plane - fast_div(plane, inv_c) * (unsigned)p.C_in);
  const int iw0 = min(seg * 4, p.W - 4);
  const int first_q = seg * 4 - iw0;
  const size_t pb = (size_t)plane * p.Ho * p.Wo;
  float am[4] = {0.f, 0.f, 0.f, 0.f}, aM[4] = {0.f, 0.f, 0.f, 0.f};
  if constexpr (S == 1) {
    float g6[3][6];
    int c6[3][6];
#pragma unroll
    for (int i = 0; i < 3; ++i) {  // input (ih, iw) is read through tap (i, j) by output (ih + ph - i, iw + pw - j)
      const int oh = ih + p.ph - i;
      const bool row_ok = (oh >= 0 && oh < p.Ho);
      const size_t rb = pb + (size_t)min(max(oh, 0), p.Ho - 1) * p.Wo;
#pragma unroll
      for (int k = 0; k < 6; ++k) {
        const int ow = iw0 + p.pw - 2 + k;
        const bool ok = row_ok && ow >= 0 && ow < p.Wo;
        const size_t o = rb + min(max(ow, 0), p.Wo - 1);
        const float g = gy[o];
        const int code = idx[o];
        g6[i][k] = ok ? g : 0.f;
        c6[i][k] = ok ? code : 0xff;  // a code no tap matches
      }
    }
    dw_gather4<MODE>(g6, c6, am, aM);
  } else if constexpr (PAR >= 0) {
    // Stride 2 with W a multiple of 4: iw0 = 4 * seg, so B = iw0 + pw has the parity PAR of pw for every lane, and
    // which taps can reach a pixel is known at compile time: a pixel q with B + q even is read through taps j = 0
    // and j = 2 of two neighbouring outputs, one with B + q odd through tap j = 1 of one output.  Likewise a row
    // ih is read through tap rows i0 = (ih + ph) & 1 and i0 + 2 only: 2 rows x 6 (tap, pixel) pairs instead of
    // 3 x 12.  Outputs ob .. ob + 2 of a row serve the lane's four pixels.
    const int B = iw0 + p.pw;
    const int ob = ((B - 2) >> 1) + PAR;
    const int i0 = (ih + p.ph) & 1;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int i = i0 + 2 * r;
      const int th = ih + p.ph - i;         // even by construction
      const bool row_ok = i < 3 && th >= 0 && (th >> 1) < p.Ho;
      const size_t rb = pb + (size_t)min(max(th >> 1, 0), p.Ho - 1) * p.Wo;
      float g3[3];
      int c3[3];
#pragma unroll
      for (int m = 0; m < 3; ++m) {
        const int ow = ob + m;
        const bool ok = row_ok && ow >= 0 && ow < p.Wo;
        const size_t o = rb + min(max(ow, 0), p.Wo - 1);
        g3[m] = gy[o];
        c3[m] = ok ? (int)idx[o] : 0xff;  // a code no tap matches
      }
      const int t0 = i * 3;  // tap (i, 0)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (((q + PAR) & 1) == 0) {  // B + q even: taps j = 0 (output m = (q + PAR) / 2 + 1 - PAR) and j = 2 (one less)
          const int m0 = (q + PAR) / 2 + 1 - PAR, m2 = m0 - 1;
          if (DO_MIN) {
            am[q] += ((c3[m0] & 15) == t0) ? g3[m0] : 0.f;
            am[q] += ((c3[m2] & 15) == t0 + 2) ? g3[m2] : 0.f;
          }
          if (DO_MAX) {
            aM[q] += ((c3[m0] >> 4) == t0) ? g3[m0] : 0.f;
            aM[q] += ((c3[m2] >> 4) == t0 + 2) ? g3[m2] : 0.f;
          }
        } else {                     // B + q odd: tap j = 1 of output m = (q + PAR + 1) / 2 - PAR
          const int m1 = (q + PAR + 1) / 2 - PAR;
          if (DO_MIN) am[q] += ((c3[m1] & 15) == t0 + 1) ? g3[m1] : 0.f;
          if (DO_MAX) aM[q] += ((c3[m1] >> 4) == t0 + 1) ? g3[m1] : 0.f;
        }
      }
    }
  } else {
    const int B = iw0 + p.pw;               // column of tap j = 0 of pixel q = 0, doubled output coordinates
    const bool odd = (B & 1) != 0;
    const int ow_base = (B - 2) >> 1;       // floor; the 4 candidate outputs of a row are ow_base .. ow_base + 3
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const int th = ih + p.ph - i;
      const bool row_ok = (th >= 0) && ((th & 1) == 0) && ((th >> 1) < p.Ho);
      const size_t rb = pb + (size_t)min(max(th >> 1, 0), p.Ho - 1) * p.Wo;
      float g4[4];
      int ce[4], co[4];  // winner bytes, kept only for the parity they can be met with
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int ow = ow_base + k;
        const bool ok = row_ok && ow >= 0 && ow < p.Wo;
        const size_t o = rb + min(max(ow, 0), p.Wo - 1);
        const float g = gy[o];
        const int code = idx[o];
        g4[k] = g;
        ce[k] = (ok && !odd) ? code : 0xff;
        co[k] = (ok && odd) ? code : 0xff;
      }
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        const int tp = i * 3 + j;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          // B + q - j even: B even and q - j even -> output ow_base + (q - j) / 2 + 1; B odd and q - j odd ->
          // output ow_base + (q - j + 3) / 2
          const bool even_pair = ((q - j) & 1) == 0;
          const int k = even_pair ? (q - j) / 2 + 1 : (q - j + 3) / 2;
          const int code = even_pair ? ce[k] : co[k];
          if (DO_MIN) am[q] += ((code & 15) == tp) ? g4[k] : 0.f;
          if (DO_MAX) aM[q] += ((code >> 4) == tp) ? g4[k] : 0.f;
        }
      }
    }
  }
  const float a = (TWO && alpha) ? alpha[c] : 1.f, b = (TWO && beta) ? beta[c] : 1.f;
  float acc[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) acc[q] = (DO_MIN ? a * am[q] : 0.f) + (DO_MAX ? b * aM[q] : 0.f);
  store_row<4>(grad_x + ((size_t)plane * p.H + ih) * p.W + iw0, acc, first_q);
}

// ------------------------------------------------------------------------------------------ backward w.r.t. x

// Generic gather, one thread per input element: tap (i, j) of output (oh, ow) reads input
// (oh*s - p + i*d, ow*s - p + j*d), so the input pixel looks, for every tap, at the one output (if any)
// that would read it through that tap and takes its gradient if that tap is the output's winner.
// SS: the stride when it is 1 or 2 on both axes (no integer division then), 0 = any stride.
template <int MODE, int SS>
__global__ __launch_bounds__(256) void dw_bwd_x_generic_kernel(Params p, int mult, const float* __restrict__ gy,
                                                               const uint8_t* __restrict__ idx,
                                                               const float* __restrict__ alpha,
                                                               const float* __restrict__ beta,
                                                               float* __restrict__ grad_x) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr bool TWO = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  const size_t total = (size_t)p.N * p.C_in * p.H * p.W;
  const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= total) return;
  const int iw = (int)(e % p.W);
  const int ih = (int)((e / p.W) % p.H);
  const int c = (int)((e / ((size_t)p.W * p.H)) % p.C_in);
  const int n = (int)(e / ((size_t)p.W * p.H * p.C_in));
  float acc = 0.f;
  for (int mm = 0; mm < mult; ++mm) {
    const int co = c * mult + mm;
    const float a = (TWO && alpha) ? alpha[co] : 1.f, b = (TWO && beta) ? beta[co] : 1.f;
    const size_t pb = ((size_t)n * p.C_out + co) * p.Ho * p.Wo;
    for (int i = 0; i < p.KH; ++i) {
      const int th = ih + p.ph - i * p.dh;
      const int sh = SS ? SS : p.sh, sw = SS ? SS : p.sw;
      if (th < 0 || th % sh != 0 || th / sh >= p.Ho) continue;
      for (int j = 0; j < p.KW; ++j) {
        const int tw = iw + p.pw - j * p.dw;
        if (tw < 0 || tw % sw != 0 || tw / sw >= p.Wo) continue;
        const size_t o = pb + (size_t)(th / sh) * p.Wo + tw / sw;
        const int code = idx[o], t = i * p.KW + j;
        const float g = gy[o];
        if (DO_MIN && (code & 15) == t) acc += a * g;
        if (DO_MAX && (code >> 4) == t) acc += b * g;
      }
    }
  }
  grad_x[e] = acc;
}

// 3x3, stride 1, dilation 1: a wave owns TH x TW INPUT pixels of one (image, input channel) plane and stages
// the gy / winner tiles of the outputs around them in LDS (gradient 0 and a code no tap matches outside
// the output plane).
template <int MODE, int TW>
__global__ __launch_bounds__(WAVES * 64) void dw_bwd_x_tiled_kernel(Params p, int mult, const float* __restrict__ gy,
                                                                    const uint8_t* __restrict__ idx,
                                                                    const float* __restrict__ alpha,
                                                                    const float* __restrict__ beta,
                                                                    const float* __restrict__ x,
                                                                    float* __restrict__ grad_x,
                                                                    float* __restrict__ grad_alpha,
                                                                    float* __restrict__ grad_beta, int tiles_h,
                                                                    unsigned inv_tiles_h, int imgs_per_wave) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr bool TWO = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  constexpr int LR = TW / 4, TH = 64 / LR;
  constexpr int ROWS = TH + 2, COLS = TW + 2;
  constexpr int CPR = (COLS + 3 + 3) / 4, PITCH = 4 * CPR;  // 4-element chunks per tile row, as in the forward kernel
  __shared__ __attribute__((aligned(16))) float g_all[WAVES][ROWS * PITCH];
  __shared__ __attribute__((aligned(16))) int c_all[WAVES][ROWS * PITCH];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int tw = blockIdx.x;
  const unsigned u = blockIdx.y * WAVES + wave;  // (input channel, tile row)
  const int c = (int)((tiles_h == 1) ? u : __umulhi(u, inv_tiles_h));
  const int th = (int)u - c * tiles_h;
  if (c >= p.C_in) return;  // whole wave; no workgroup barrier
  const int own_w = tw * TW;
  const int org_w = min(own_w, max(p.W - TW, 0));
  const int ih0 = th * TH;
  float* const gt = g_all[wave];
  int* const ct = c_all[wave];

  const int r = lane / LR, seg = lane % LR;
  const int ih = ih0 + r;
  const int nominal = org_w + 4 * seg;
  const int lo = max(own_w, nominal);
  const int iw0 = min(nominal, p.W - 4);
  const int first_q = lo - iw0;
  const bool act = (ih < p.H) && (first_q < 4);

  // tile row rr holds output row oh_base + rr, tile column cc output column cbase + cc (cbase a multiple of
  // 4, or -4); input (ih, iw) is read through tap (i, j) by output (ih + ph - i, iw + pw - j)
  const int oh_base = ih0 + p.ph - 2, ow_base = org_w + p.pw - 2;
  const int cbase = (ow_base < 0) ? -4 : (ow_base & ~3);
  const int dd = (4 - (p.Wo & 3)) & 3;
  const int lc = iw0 + p.pw - 2 - cbase;  // tile column of output column iw0 + pw - 2
  // The wave walks the same tile through imgs_per_wave images, so that the x part of the coefficient
  // gradients (one value per output channel) leaves it with ONE atomic per branch instead of one per image:
  // atomics to the same address are served one after the other.
  const bool want_coef = TWO && x && (grad_alpha || grad_beta);
  float sx_min = 0.f, sx_max = 0.f;
  const int n_first = blockIdx.z * imgs_per_wave, n_last = min(n_first + imgs_per_wave, p.N);
  for (int n = n_first; n < n_last; ++n) {
  const int plane = n * p.C_in + c;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int mm = 0; mm < mult; ++mm) {
    const int co = c * mult + mm;
    const size_t pb = ((size_t)n * p.C_out + co) * p.Ho * p.Wo;
    wave_lds_fence();  // every lane is done with the tiles of the previous output channel
    // chunks of 4 outputs (16 bytes of gy, 4 bytes of winners), all in flight before the first LDS write; a
    // chunk that hangs over the row end is loaded from Wo - 4 and shifted by dd
    constexpr int NCH = ROWS * CPR, NIT = (NCH + 63) / 64;
    f4u sg[NIT];
    unsigned sc[NIT];
#pragma unroll
    for (int k = 0; k < NIT; ++k) {
      const int e = min(lane + 64 * k, NCH - 1);
      const int rr = e / CPR, q = e - rr * CPR;
      const int oh = min(max(oh_base + rr, 0), p.Ho - 1);
      const int start = min(max(cbase + 4 * q, 0), p.Wo - 4);
      const size_t o = pb + (size_t)oh * p.Wo + start;
      sg[k] = *(const f4u*)(gy + o);
      sc[k] = *(const u1a*)(idx + o);
    }
#pragma unroll
    for (int k = 0; k < NIT; ++k) {
      const int e = lane + 64 * k;
      const int rr = e / CPR, q = e - rr * CPR;
      const int oh = oh_base + rr, c0 = cbase + 4 * q;
      const bool row_ok = (oh >= 0 && oh < p.Ho);
      f4u v = sg[k];
      unsigned cw = sc[k];
      if (dd != 0 && c0 + 4 > p.Wo) {
        const f4u u = v;
        if (dd == 1) { v.x = u.y; v.y = u.z; v.z = u.w; }
        else if (dd == 2) { v.x = u.z; v.y = u.w; }
        else { v.x = u.w; }
        cw >>= 8 * dd;
      }
      const bool k0 = row_ok && c0 >= 0 && c0 < p.Wo, k1 = row_ok && c0 >= 0 && c0 + 1 < p.Wo;
      const bool k2 = row_ok && c0 >= 0 && c0 + 2 < p.Wo, k3 = row_ok && c0 >= 0 && c0 + 3 < p.Wo;
      f4a go;
      i4a co4;
      go.x = k0 ? v.x : 0.f; co4.x = k0 ? (int)(cw & 0xffu) : 0xff;   // 0xff: a code no tap matches
      go.y = k1 ? v.y : 0.f; co4.y = k1 ? (int)((cw >> 8) & 0xffu) : 0xff;
      go.z = k2 ? v.z : 0.f; co4.z = k2 ? (int)((cw >> 16) & 0xffu) : 0xff;
      go.w = k3 ? v.w : 0.f; co4.w = k3 ? (int)(cw >> 24) : 0xff;
      if (e < NCH) {
        *(f4a*)&gt[rr * PITCH + 4 * q] = go;
        *(i4a*)&ct[rr * PITCH + 4 * q] = co4;
      }
    }
    wave_lds_fence();
    const float a = (TWO && alpha) ? alpha[co] : 1.f, b = (TWO && beta) ? beta[co] : 1.f;
    float am[4] = {0.f, 0.f, 0.f, 0.f}, aM[4] = {0.f, 0.f, 0.f, 0.f};  // unscaled gradient through each branch
    float g6[3][6];
    int c6[3][6];
#pragma unroll
    for (int i = 0; i < 3; ++i) {  // outputs of tile row r + 2 - i, tile columns lc .. lc + 5
      lds_run<6>(g6[i], &gt[(r + 2 - i) * PITCH + lc]);
      lds_run<6>((float*)c6[i], (const float*)&ct[(r + 2 - i) * PITCH + lc]);
    }
    dw_gather4<MODE>(g6, c6, am, aM);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (DO_MIN) acc[q] += a * am[q];
      if (DO_MAX) acc[q] += b * aM[q];
    }
    // The x part of the coefficient gradients: sum over outputs of gy * x[winner] = sum over input pixels of
    // x * (gradient that reached the pixel through that branch).  Pixels this lane computes for a neighbour
    // (moved last segment / tile) are left to their owner.
    if (want_coef) {
      if (act) {
        const f4u xv = *(const f4u*)(x + ((size_t)plane * p.H + ih) * p.W + iw0);
        const float x4[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (q >= first_q) { sx_min += x4[q] * am[q]; sx_max += x4[q] * aM[q]; }
      }
      if (mult > 1 || n == n_last - 1) {  // several output channels per input channel: one flush per channel and image
        const float sa = wave_sum(sx_min), sb = wave_sum(sx_max);
        if (lane == 0) {
          if (grad_alpha) atomicAdd(grad_alpha + co, sa);
          if (grad_beta) atomicAdd(grad_beta + co, sb);
        }
        sx_min = sx_max = 0.f;
      }
    }
  }
  if (act && grad_x) store_row<4>(grad_x + ((size_t)plane * p.H + ih) * p.W + iw0, acc, first_q);
  }
}

// ------------------------------------------------------------------------------------------ parameter gradients

// grad_w_b[co, t] = coef_b * S_b[t], S_b[t] = sum of gy over the outputs of channel co whose branch-b winner is
// tap t; grad_alpha[co] = sum gy * m and grad_beta[co] = sum gy * M, where the branch output at the winner
// is x[winner] + w[t], so the sum splits into sum gy * x[winner] plus sum over t of w[t] * S_b[t] (the
// second part comes from the tap sums; the split differs from the rounded x + w by one rounding per term).
// The tiled input-gradient kernel adds the x part itself (it has every input pixel's share of the gradient in
// registers); this kernel then only adds the w part (gather_x == 0).
// Workgroup = (output channel, slice of the batch).  Every thread keeps its own column of partial sums in
// LDS (bins[row][thread]: no conflicts, no atomics), rows: KK taps per branch, then one for sum gy * x.
// A thread takes 4 consecutive outputs per trip (one 16-byte and one 4-byte load) and fetches the next
// trip's operands before it works on the current ones.
template <int MODE>
__global__ __launch_bounds__(256) void dw_bwd_params_kernel(Params p, int mult, const float* __restrict__ x,
                                                            const float* __restrict__ w_min,
                                                            const float* __restrict__ w_max,
                                                            const float* __restrict__ alpha,
                                                            const float* __restrict__ beta,
                                                            const float* __restrict__ gy,
                                                            const uint8_t* __restrict__ idx,
                                                            float* __restrict__ grad_w_min,
                                                            float* __restrict__ grad_w_max,
                                                            float* __restrict__ grad_alpha,
                                                            float* __restrict__ grad_beta, int n_per_block,
                                                            int gather_x) {
  constexpr bool DO_MIN = (MODE != TCONV_MAX), DO_MAX = (MODE != TCONV_MIN);
  constexpr bool TWO = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  constexpr int NBR = TWO ? 2 : 1;
  constexpr int NT = 256, PITCH = NT + 1;
  HIP_DYNAMIC_SHARED(float, bins)  // [NBR * (KK + 1)][PITCH], then int toff[16]
  const int KK = p.KH * p.KW;
  const int rows = NBR * (KK + 1);
  int* const toff = (int*)(bins + rows * PITCH);  // offset of tap t from the window's first input pixel
  const int co = blockIdx.x, c = co / mult;
  const int n0 = blockIdx.y * n_per_block;
  const int n1 = min(n0 + n_per_block, p.N);
  const int tid = threadIdx.x;
  if (tid < 16) {
    const int t = min(tid, KK - 1), i = t / p.KW, j = t - i * p.KW;
    toff[tid] = i * p.dh * p.W + j * p.dw;
  }
  for (int rw = 0; rw < rows; ++rw) bins[rw * PITCH + tid] = 0.f;
  __syncthreads();
  const bool want_coef = TWO && (grad_alpha || grad_beta);
  const bool want_x = want_coef && gather_x;  // else the input-gradient kernel has added the x part already
  const int plane = p.Ho * p.Wo, xplane = p.H * p.W;
  const int ngrp = plane >> 2;                 // groups of 4 consecutive outputs inside a plane
  const int base_max = (NBR - 1) * (KK + 1);   // first row of the max-plus branch
  float sx_min = 0.f, sx_max = 0.f;            // sum gy * x[winner]

  // one output: g, its winner byte, its position, its image's input plane
  auto one = [&](float g, int code, int oh, int ow, const float* xp) {
    const int first = (oh * p.sh - p.ph) * p.W + (ow * p.sw - p.pw);  // may lie in the padding; the winner does not
    if (DO_MIN) {
      const int t = min(code & 15, KK - 1);
      bins[t * PITCH + tid] += g;
      if (want_x) sx_min += g * xp[min(max(first + toff[t], 0), xplane - 1)];  // clamp: a corrupted index stays in bounds
    }
    if (DO_MAX) {
      const int t = min(code >> 4, KK - 1);
      bins[(base_max + t) * PITCH + tid] += g;
      if (want_x) sx_max += g * xp[min(max(first + toff[t], 0), xplane - 1)];
    }
  };

  if (ngrp > 0) {
    const int total = (n1 - n0) * ngrp;  // trips of the slice, n-major
    auto fetch = [&](int f, f4u& g4, unsigned& c4, int& n, int& pix) {
      n = n0 + f / ngrp;
      pix = (f - (n - n0) * ngrp) * 4;
      const size_t o = ((size_t)n * p.C_out + co) * plane + pix;
      g4 = *(const f4u*)(gy + o);
      c4 = *(const u1a*)(idx + o);
    };
    int f = tid;
    f4u g4 = {0.f, 0.f, 0.f, 0.f};
    unsigned c4 = 0;
    int n = n0, pix = 0;
    if (f < total) fetch(f, g4, c4, n, pix);
    while (f < total) {
      const int fn = f + NT;
      f4u g4n = g4;
      unsigned c4n = c4;
      int nn = n, pixn = pix;
      if (fn < total) fetch(fn, g4n, c4n, nn, pixn);
      const float* xp = want_x ? x + ((size_t)n * p.C_in + c) * xplane : nullptr;
      int oh = pix / p.Wo, ow = pix - oh * p.Wo;
      const float gs[4] = {g4.x, g4.y, g4.z, g4.w};
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        one(gs[u], (int)((c4 >> (8 * u)) & 0xffu), oh, ow, xp);
        if (++ow == p.Wo) { ow = 0; ++oh; }
      }
      g4 = g4n; c4 = c4n; n = nn; pix = pixn; f = fn;
    }
  }
  // the last plane % 4 outputs of every plane
  const int rem = plane - 4 * ngrp;
  for (int e = tid; e < (n1 - n0) * rem; e += NT) {
    const int n = n0 + e / rem, pix = 4 * ngrp + e % rem;
    const size_t o = ((size_t)n * p.C_out + co) * plane + pix;
    const float* xp = want_x ? x + ((size_t)n * p.C_in + c) * xplane : nullptr;
    one(gy[o], idx[o], pix / p.Wo, pix % p.Wo, xp);
  }
  if (want_x) {
    if (DO_MIN) bins[KK * PITCH + tid] = sx_min;
    if (DO_MAX) bins[(base_max + KK) * PITCH + tid] = sx_max;
  }
  __syncthreads();
  // one thread per row adds the 256 partial sums in double; row KK of a branch becomes its coefficient sum
  double* const tot = (double*)(((uintptr_t)(toff + 16) + 7) & ~(uintptr_t)7);  // [rows]
  if (tid < rows) {
    double sacc = 0.0;
    for (int k = 0; k < NT; ++k) sacc += (double)bins[tid * PITCH + k];
    tot[tid] = sacc;
  }
  __syncthreads();
  if (tid < rows) {
    const int br = tid / (KK + 1), k = tid - br * (KK + 1);
    const bool is_max = DO_MAX && (NBR == 1 || br == 1);
    if (k < KK) {
      const float coef = !TWO ? 1.f : (is_max ? (beta ? beta[co] : 1.f) : (alpha ? alpha[co] : 1.f));
      float* gw = is_max ? grad_w_max : grad_w_min;
      if (gw) atomicAdd(gw + (size_t)co * KK + k, (float)((double)coef * tot[tid]));
    } else if (want_coef) {
      float* gc = is_max ? grad_beta : grad_alpha;
      const float* wv = (is_max ? w_max : w_min) + (size_t)co * KK;
      double sacc = want_x ? tot[tid] : 0.0;
      for (int t = 0; t < KK; ++t) sacc += (double)wv[t] * tot[br * (KK + 1) + t];
      if (gc) atomicAdd(gc + co, (float)sacc);
    }
  }
}

// Zero fill of the (small) parameter gradients before the atomics: up to four buffers in one launch, as a
// kernel so that the call can sit in a captured graph.
struct ZeroList {
  float* ptr[4];
  unsigned n[4];
};

__global__ __launch_bounds__(256) void dw_fill_zero_kernel(ZeroList z) {
  const unsigned stride = gridDim.x * blockDim.x;
#pragma unroll
  for (int b = 0; b < 4; ++b)
    for (unsigned i = blockIdx.x * blockDim.x + threadIdx.x; i < z.n[b]; i += stride) z.ptr[b][i] = 0.f;
}

int resident_cus() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    cus = 256;
  return cus;
}

bool force_generic() {
  const char* e = getenv("TCONV_FORWARD_KERNEL");
  return e && strcmp(e, "generic") == 0;
}

// widest tile (a multiple of 4 columns, at most 32) that a row of `width` pixels fills reasonably
int tile_width(int width) { return width > 16 ? 32 : (width > 8 ? 16 : 8); }

// Launch grid of the tiled kernels: x = tile column, y = ceil(channels * tiles_h / WAVES) (a workgroup's waves
// take consecutive (channel, tile row) pairs), z = image.  inv_tiles_h = floor(2^32 / tiles_h) + 1 turns the
// split of a pair number u into a multiply-high (exact while u * tiles_h < 2^32; u < 2^18 * tiles_h here).
struct TileGrid {
  dim3 grid;
  unsigned inv_tiles_h;
};

TileGrid tile_grid(int tiles_w, int tiles_h, int channels, int images) {
  TileGrid t;
  const long long pairs = (long long)channels * tiles_h;
  t.grid = dim3((unsigned)tiles_w, (unsigned)((pairs + WAVES - 1) / WAVES), (unsigned)images);
  t.inv_tiles_h = tiles_h > 1 ? (unsigned)(0x100000000ull / (unsigned)tiles_h) + 1u : 0u;
  return t;
}

// the tiled kernels put channel and image into grid dimensions y and z and address a plane with 32 bits
bool tiled_dims_ok(const Params& p) {
  // grid y = channels * tile rows / WAVES <= 65535; tile rows <= H / 8 + 1
  const long long worst = ((long long)(p.C_out > p.C_in ? p.C_out : p.C_in) * (p.H / 8 + 1) + WAVES - 1) / WAVES;
  return worst <= 65535 && p.N <= 65535 && (long long)p.H * p.W < (1 << 24) && (long long)p.N * p.C_out < 0x7fffffffLL;
}

bool fwd_tiled_ok(const Params& p) {
  if (p.KH != 3 || p.KW != 3 || p.dh != 1 || p.dw != 1) return false;
  if (p.sh != p.sw || (p.sh != 1 && p.sh != 2)) return false;
  return tiled_dims_ok(p) && p.Wo >= 8;
}

bool bwd_x_tiled_ok(const Params& p) {
  return p.KH == 3 && p.KW == 3 && p.dh == 1 && p.dw == 1 && p.sh == 1 && p.sw == 1 && p.W >= 8 &&
         tiled_dims_ok(p);
}

// The by-rows kernels: 3x3, dilation 1, one input channel per output channel, rows of at least 4 pixels, and
// row numbers small enough for the multiply-high quotients (u * d < 2^32 for d = segments, rows, channels).
bool rows_dims_ok(long long planes, int rows, int width, int channels) {
  if (width < 4) return false;
  const long long segs = (width + 3) / 4, units = planes * rows * segs;
  const long long dmax = segs > rows ? (segs > channels ? segs : channels) : (rows > channels ? rows : channels);
  return units * dmax < 0xffffffffLL && units + 256 < 0xffffffffLL;
}

bool fwd_rows_ok(const Params& p) {
  if (p.KH != 3 || p.KW != 3 || p.dh != 1 || p.dw != 1 || p.C_out != p.C_in) return false;
  if (p.sh != p.sw || (p.sh != 1 && p.sh != 2)) return false;
  return rows_dims_ok((long long)p.N * p.C_out, p.Ho, p.Wo, p.C_out);
}

bool bwd_x_rows_ok(const Params& p) {
  if (p.KH != 3 || p.KW != 3 || p.dh != 1 || p.dw != 1 || p.C_out != p.C_in) return false;
  if (p.sh != p.sw || (p.sh != 1 && p.sh != 2)) return false;
  return rows_dims_ok((long long)p.N * p.C_in, p.H, p.W, p.C_in);
}

// a plane that fills at most half of a wave's tile goes by rows
bool small_plane(int rows, int width) { return (long long)rows * (tile_width(width) / 4) <= 32; }

unsigned inv_of(int d) { return d > 1 ? (unsigned)(0x100000000ull / (unsigned)d) + 1u : 0u; }

// 0: generic, 1: tiled through LDS, 2: by rows
int fwd_kernel_choice(const Params& p) {
  if (force_generic()) return 0;
  const bool tiled = fwd_tiled_ok(p), rows = fwd_rows_ok(p);
  if (rows && (!tiled || small_plane(p.Ho, p.Wo))) return 2;
  return tiled ? 1 : 0;
}

int bwd_x_kernel_choice(const Params& p) {
  if (force_generic()) return 0;
  const bool tiled = bwd_x_tiled_ok(p), rows = bwd_x_rows_ok(p);
  if (rows && (!tiled || small_plane(p.H, p.W))) return 2;
  return tiled ? 1 : 0;
}

template <int MODE, int S>
hipError_t launch_fwd_rows(const Params& p, const DwArgs& a, hipStream_t s) {
  const int segs = (p.Wo + 3) / 4;
  const unsigned n_units = (unsigned)((long long)p.N * p.C_out * p.Ho * segs);
  const dim3 grid((n_units + 255) / 256);
  if (a.idx)
    hipLaunchKernelGGL((dw_fwd_rows_kernel<MODE, S, true>), grid, dim3(256), 0, s, p, a.x, a.w_min, a.w_max, a.alpha,
                       a.beta, a.y, a.idx, segs, n_units, inv_of(segs), inv_of(p.Ho), inv_of(p.C_out));
  else
    hipLaunchKernelGGL((dw_fwd_rows_kernel<MODE, S, false>), grid, dim3(256), 0, s, p, a.x, a.w_min, a.w_max, a.alpha,
                       a.beta, a.y, a.idx, segs, n_units, inv_of(segs), inv_of(p.Ho), inv_of(p.C_out));
  return hipGetLastError();
}

template <int MODE, int S, int TW>
hipError_t launch_fwd_tile(const Params& p, int mult, const DwArgs& a, hipStream_t s) {
  constexpr int TH = 64 / (TW / 4);
  const int tiles_w = (p.Wo + TW - 1) / TW, tiles_h = (p.Ho + TH - 1) / TH;
  const TileGrid tg = tile_grid(tiles_w, tiles_h, p.C_out, p.N);
  if (a.idx)
    hipLaunchKernelGGL((dw_fwd_tiled_kernel<MODE, S, TW, true>), tg.grid, dim3(WAVES * 64), 0, s, p, mult, a.x,
                       a.w_min, a.w_max, a.alpha, a.beta, a.y, a.idx, tiles_h, tg.inv_tiles_h);
  else
    hipLaunchKernelGGL((dw_fwd_tiled_kernel<MODE, S, TW, false>), tg.grid, dim3(WAVES * 64), 0, s, p, mult, a.x,
                       a.w_min, a.w_max, a.alpha, a.beta, a.y, a.idx, tiles_h, tg.inv_tiles_h);
  return hipGetLastError();
}

template <int MODE, int S>
hipError_t launch_fwd_s(const Params& p, int mult, const DwArgs& a, hipStream_t s) {
  switch (tile_width(p.Wo)) {
    case 32: return launch_fwd_tile<MODE, S, 32>(p, mult, a, s);
    case 16: return launch_fwd_tile<MODE, S, 16>(p, mult, a, s);
    default: return launch_fwd_tile<MODE, S, 8>(p, mult, a, s);
  }
}

template <int MODE>
hipError_t launch_fwd(const Params& p, const DwArgs& a, hipStream_t s) {
  const int mult = p.C_out / p.C_in;
  if (fwd_kernel_choice(p) == 2)
    return p.sh == 1 ? launch_fwd_rows<MODE, 1>(p, a, s) : launch_fwd_rows<MODE, 2>(p, a, s);
  if (fwd_kernel_choice(p) == 1)
    return p.sh == 1 ? launch_fwd_s<MODE, 1>(p, mult, a, s) : launch_fwd_s<MODE, 2>(p, mult, a, s);
  const size_t total = (size_t)p.N * p.C_out * p.Ho * p.Wo;
  hipLaunchKernelGGL(dw_fwd_generic_kernel<MODE>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, p, mult,
                     a.x, a.w_min, a.w_max, a.alpha, a.beta, a.y, a.idx);
  return hipGetLastError();
}

template <int MODE, int TW>
hipError_t launch_bwd_x_tile(const Params& p, int mult, const DwArgs& a, const DwGrads& g, bool want_coef,
                             hipStream_t s) {
  constexpr int TH = 64 / (TW / 4);
  const int tiles_w = (p.W + TW - 1) / TW, tiles_h = (p.H + TH - 1) / TH;
  // images per wave: as many as still leave about four waves per SIMD slot busy, at most 8 (measured: 4 - 8
  // is the flat optimum; one costs twice the time in atomics, 32 starves the chip of waves)
  const long long waves_per_image = (long long)tiles_w * tiles_h * p.C_in;
  int ipw = 1;
  if (want_coef) {
    ipw = (int)((waves_per_image * p.N) / (4LL * 4 * resident_cus()));
    ipw = ipw < 1 ? 1 : (ipw > 8 ? 8 : ipw);
    if (const char* e = getenv("TCONV_DW_IPW")) ipw = atoi(e) > 0 ? atoi(e) : ipw;  // tuning aid
  }
  const TileGrid tg = tile_grid(tiles_w, tiles_h, p.C_in, (p.N + ipw - 1) / ipw);
  hipLaunchKernelGGL((dw_bwd_x_tiled_kernel<MODE, TW>), tg.grid, dim3(WAVES * 64), 0, s, p, mult, g.gy, a.idx,
                     a.alpha, a.beta, want_coef ? a.x : nullptr, g.grad_x, g.grad_alpha, g.grad_beta, tiles_h,
                     tg.inv_tiles_h, ipw);
  return hipGetLastError();
}

template <int MODE>
hipError_t launch_bwd(const Params& p, const DwArgs& a, const DwGrads& g, hipStream_t s) {
  constexpr bool TWO = (MODE == TCONV_COMPOUND || MODE == TCONV_PARALLEL);
  const int mult = p.C_out / p.C_in, KK = p.KH * p.KW;
  float* gmin = g.grad_w_min;
  float* gmax = g.grad_w_max;
  if (MODE == TCONV_COMPOUND) gmin = gmax = (g.grad_w_min ? g.grad_w_min : g.grad_w_max);
  const bool want_coef = TWO && (g.grad_alpha || g.grad_beta);
  const bool want_params = (MODE != TCONV_MAX && gmin) || (MODE != TCONV_MIN && gmax) || want_coef;
  if (want_params) {  // every parameter gradient is accumulated with atomics
    const unsigned nw = (unsigned)p.C_out * KK;
    ZeroList z = {{nullptr, nullptr, nullptr, nullptr}, {0u, 0u, 0u, 0u}};
    int nz = 0;
    auto add = [&](float* ptr, unsigned n) { if (ptr) { z.ptr[nz] = ptr; z.n[nz] = n; ++nz; } };
    if (MODE != TCONV_MAX) add(gmin, nw);
    if (MODE == TCONV_MAX || MODE == TCONV_PARALLEL) add(gmax, nw);
    add(g.grad_alpha, (unsigned)p.C_out);
    add(g.grad_beta, (unsigned)p.C_out);
    unsigned zblocks = (nw + 255) / 256;
    if (zblocks > 1024) zblocks = 1024;
    hipLaunchKernelGGL(dw_fill_zero_kernel, dim3(zblocks), dim3(256), 0, s, z);
  }
  const int choice = bwd_x_kernel_choice(p);
  const bool tiled = choice == 1;
  if (choice == 2 && g.grad_x) {
    const int segs = (p.W + 3) / 4;
    const unsigned n_units = (unsigned)((long long)p.N * p.C_in * p.H * segs);
    if (p.sh == 1)
      hipLaunchKernelGGL((dw_bwd_x_rows_kernel<MODE, 1>), dim3((n_units + 255) / 256), dim3(256), 0, s, p, g.gy, a.idx,
                         a.alpha, a.beta, g.grad_x, segs, n_units, inv_of(segs), inv_of(p.H), inv_of(p.C_in));
    else if (p.W % 4 == 0 && (p.pw & 1) == 0)  // every lane's first column has the parity of pad_w
      hipLaunchKernelGGL((dw_bwd_x_rows_kernel<MODE, 2, 0>), dim3((n_units + 255) / 256), dim3(256), 0, s, p, g.gy, a.idx,
                         a.alpha, a.beta, g.grad_x, segs, n_units, inv_of(segs), inv_of(p.H), inv_of(p.C_in));
    else if (p.W % 4 == 0)
      hipLaunchKernelGGL((dw_bwd_x_rows_kernel<MODE, 2, 1>), dim3((n_units + 255) / 256), dim3(256), 0, s, p, g.gy, a.idx,
                         a.alpha, a.beta, g.grad_x, segs, n_units, inv_of(segs), inv_of(p.H), inv_of(p.C_in));
    else
      hipLaunchKernelGGL((dw_bwd_x_rows_kernel<MODE, 2>), dim3((n_units + 255) / 256), dim3(256), 0, s, p, g.gy, a.idx,
                         a.alpha, a.beta, g.grad_x, segs, n_units, inv_of(segs), inv_of(p.H), inv_of(p.C_in));
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  } else if (tiled && (g.grad_x || want_coef)) {  // grad_x and the x part of the coefficient gradients
    hipError_t e;
    switch (tile_width(p.W)) {
      case 32: e = launch_bwd_x_tile<MODE, 32>(p, mult, a, g, want_coef, s); break;
      case 16: e = launch_bwd_x_tile<MODE, 16>(p, mult, a, g, want_coef, s); break;
      default: e = launch_bwd_x_tile<MODE, 8>(p, mult, a, g, want_coef, s); break;
    }
    if (e != hipSuccess) return e;
  } else if (g.grad_x) {
    const size_t total = (size_t)p.N * p.C_in * p.H * p.W;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (p.sh == p.sw && p.sh == 1)
      hipLaunchKernelGGL((dw_bwd_x_generic_kernel<MODE, 1>), grid, dim3(256), 0, s, p, mult, g.gy, a.idx, a.alpha, a.beta,
                         g.grad_x);
    else if (p.sh == p.sw && p.sh == 2)
      hipLaunchKernelGGL((dw_bwd_x_generic_kernel<MODE, 2>), grid, dim3(256), 0, s, p, mult, g.gy, a.idx, a.alpha, a.beta,
                         g.grad_x);
    else
      hipLaunchKernelGGL((dw_bwd_x_generic_kernel<MODE, 0>), grid, dim3(256), 0, s, p, mult, g.gy, a.idx, a.alpha, a.beta,
                         g.grad_x);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (want_params) {
    int slices = (2048 + p.C_out - 1) / p.C_out;  // enough workgroups to fill the chip
    if (slices > p.N) slices = p.N;
    if (slices > 65535) slices = 65535;
    const int n_per_block = (p.N + slices - 1) / slices;
    const dim3 grid((unsigned)p.C_out, (unsigned)((p.N + n_per_block - 1) / n_per_block));
    constexpr int NBR = TWO ? 2 : 1;
    const size_t lds = (size_t)NBR * (KK + 1) * 257 * sizeof(float) + 16 * sizeof(int) + (size_t)NBR * (KK + 1) * sizeof(double) + 8;
    hipLaunchKernelGGL(dw_bwd_params_kernel<MODE>, grid, dim3(256), lds, s, p, mult, a.x, a.w_min, a.w_max, a.alpha,
                       a.beta, g.gy, a.idx, gmin, gmax, g.grad_alpha, g.grad_beta, n_per_block, tiled ? 0 : 1);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_depthwise_forward(const Params& p, const DwArgs& a, hipStream_t s) {
  switch (p.mode) {
    case TCONV_MAX: return launch_fwd<TCONV_MAX>(p, a, s);
    case TCONV_MIN: return launch_fwd<TCONV_MIN>(p, a, s);
    case TCONV_COMPOUND: return launch_fwd<TCONV_COMPOUND>(p, a, s);
    default: return launch_fwd<TCONV_PARALLEL>(p, a, s);
  }
}

hipError_t launch_depthwise_backward(const Params& p, const DwArgs& a, const DwGrads& g, hipStream_t s) {
  switch (p.mode) {
    case TCONV_MAX: return launch_bwd<TCONV_MAX>(p, a, g, s);
    case TCONV_MIN: return launch_bwd<TCONV_MIN>(p, a, g, s);
    case TCONV_COMPOUND: return launch_bwd<TCONV_COMPOUND>(p, a, g, s);
    default: return launch_bwd<TCONV_PARALLEL>(p, a, g, s);
  }
}

const char* depthwise_forward_kernel_name(const Params& p) {
  const int k = fwd_kernel_choice(p);
  return k == 2 ? "dw_rows3x3" : (k == 1 ? "dw_tiled3x3" : "dw_generic");
}

}  // namespace tconv
