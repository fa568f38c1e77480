/*
 * CPU oracle for the Sum-channel tropical convolution layers.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow loop nest
 * written from the paper's layer equations.  Only the tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.  It shares no code, header,
 * table or helper with the HIP library.
 *
 * What it computes.  Base operators (paper Sec. 3.1): for one input channel,
 *   MinPlus2d(X, W, h, w, c_in, c_out) = min over the KH x KW window of X[h+i, w+j, c_in] + W[i, j, c_in, c_out]
 *   MaxPlus2d likewise with max.
 * Layers (i) MinPlus-Sum-Conv2d and (ii) MaxPlus-Sum-Conv2d sum the base operator over c_in.
 * The compound and parallel layers (Sec. 3.5 "Compound tropical convolution layers", Sec. 3.6
 * "Parallel tropical convolution layers", the ...SumConv2d2p equations):
 *   Y[h, w, c_out] = sum over c_in of ( alpha[c_in, c_out] * MinPlus2d(X, W1, ...) + beta[c_in, c_out] * MaxPlus2d(X, W2, ...) )
 * with W1 == W2 in the compound layer (one shared add feeds both, closing remark of Sec. 3.5).
 *
 * Readings where the paper is silent:
 *   - tensors are NCHW / OIHW, contiguous; alpha, beta are [C_in, C_out] (index c_in*C_out + c_out,
 *     as the paper subscripts them), NULL meaning all ones; they are not used in the single-branch
 *     layers (i), (ii);
 *   - padding holds the semiring identity, i.e. a padded tap is skipped (every window keeps at
 *     least one valid tap because pad <= dil*(k-1));
 *   - window ties keep the lowest tap index t = i*KW + j (strict compare while t ascends);
 *   - each x + w is one rounded fp32 add; a channel's term is fl(fl(alpha*m) + fl(beta*M)) (no fused
 *     multiply-add; just m or M in the single-branch layers); the channel sum starts at +0 and adds
 *     the terms in ascending c_in, each add rounded to fp32;
 *   - backward is the sub-gradient through the single winner of every (c_in, c_out, pixel) window:
 *     with g = gy[n, c_out, oh, ow],
 *       grad_x[n, c, ih*, iw*] += alpha*g (min winner) and += beta*g (max winner),
 *       grad_w1[c_out, c, i*, j*] += alpha*g, grad_w2 likewise with beta (compound: both into one tensor),
 *       grad_alpha[c, c_out] += g*m, grad_beta[c, c_out] += g*M;
 *     sums are kept in double so this side is the better-rounded one.
 *   - the one-parameter layers (beta = 1 - alpha) are this layer with that beta; their gradient
 *     is grad_alpha - grad_beta.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct oracle_shape {
  int32_t N, C_in, H, W;
  int32_t C_out, KH, KW;
  int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
} oracle_shape;

enum { ORACLE_MAX = 0, ORACLE_MIN = 1, ORACLE_COMPOUND = 2, ORACLE_PARALLEL = 3 };

/* 1 if some window of one axis has no tap inside the input (written out: every output position, every tap).  The
 * extremum of Sec. 3.1 over an empty set of taps is not defined, so such a layer is rejected. */
static int axis_has_empty_window(long in, long k, long stride, long pad, long dil, long out) {
  for (long o = 0; o < out; ++o) {
    int hit = 0;
    for (long t = 0; t < k; ++t) {
      long i = o * stride - pad + t * dil;
      if (i >= 0 && i < in) hit = 1;
    }
    if (!hit) return 1;
  }
  return 0;
}

static int out_shape(const oracle_shape* s, int32_t* H_out, int32_t* W_out) {
  long eh = (long)s->dil_h * (s->KH - 1) + 1, ew = (long)s->dil_w * (s->KW - 1) + 1;
  long nh = (long)s->H + 2L * s->pad_h - eh, nw = (long)s->W + 2L * s->pad_w - ew;
  if (nh < 0 || nw < 0) return -1;
  if (s->pad_h > eh - 1 || s->pad_w > ew - 1) return -1; /* a window could be all padding */
  *H_out = (int32_t)(nh / s->stride_h + 1);
  *W_out = (int32_t)(nw / s->stride_w + 1);
  if (axis_has_empty_window(s->H, s->KH, s->stride_h, s->pad_h, s->dil_h, *H_out) ||
      axis_has_empty_window(s->W, s->KW, s->stride_w, s->pad_w, s->dil_w, *W_out))
    return -1;
  return 0;
}

/* Base operator for one (n, c_in, c_out, oh, ow): extremum of x + w over the valid taps of the window
 * and the lowest tap index t = i*KW + j that attains it.  x_c: the H x W plane, w_cc: the KH x KW kernel. */
static void base_op(const oracle_shape* s, const float* x_c, const float* w_cc, int oh, int ow,
                    int want_max, float* best_out, int32_t* tap_out) {
  float best = 0.0f;
  int32_t bt = -1;
  for (int i = 0; i < s->KH; ++i) {
    int ih = oh * s->stride_h - s->pad_h + i * s->dil_h;
    if (ih < 0 || ih >= s->H) continue;
    for (int j = 0; j < s->KW; ++j) {
      int iw = ow * s->stride_w - s->pad_w + j * s->dil_w;
      if (iw < 0 || iw >= s->W) continue;
      volatile float sum = x_c[(size_t)ih * s->W + iw] + w_cc[i * s->KW + j];
      float v = sum;
      if (bt < 0 || (want_max ? (v > best) : (v < best))) {
        best = v;
        bt = i * s->KW + j;
      }
    }
  }
  *best_out = best;
  *tap_out = bt;
}

static float coef(const float* a, const oracle_shape* s, int c, int co) {
  return a ? a[(size_t)c * s->C_out + co] : 1.0f;
}

/*
 * Forward.  mode: MIN -> layer (i), MAX -> layer (ii), COMPOUND / PARALLEL -> the two-parameter
 * layers.  w_min is W1 (min-plus kernel), w_max is W2; compound uses w_min if non-NULL else w_max
 * for both.  y [N, C_out, H_out, W_out] fp32.
 */
int oracle_tsum_forward(const oracle_shape* s, int mode, const float* x, const float* w_min,
                        const float* w_max, const float* alpha, const float* beta, float* y) {
  int32_t Ho, Wo;
  if (out_shape(s, &Ho, &Wo) != 0) return -1;
  const int do_min = (mode != ORACLE_MAX), do_max = (mode != ORACLE_MIN);
  const int two = (mode == ORACLE_COMPOUND || mode == ORACLE_PARALLEL);
  if (mode == ORACLE_COMPOUND) w_min = w_max = (w_min ? w_min : w_max);
  if (!x || !y || (do_min && !w_min) || (do_max && !w_max)) return -1;
  const size_t KK = (size_t)s->KH * s->KW, HW = (size_t)s->H * s->W;
  for (int n = 0; n < s->N; ++n)
    for (int co = 0; co < s->C_out; ++co)
      for (int oh = 0; oh < Ho; ++oh)
        for (int ow = 0; ow < Wo; ++ow) {
          volatile float acc = 0.0f;
          for (int c = 0; c < s->C_in; ++c) {
            const float* x_c = x + ((size_t)n * s->C_in + c) * HW;
            float m = 0.0f, M = 0.0f;
            int32_t t;
            if (do_min) base_op(s, x_c, w_min + ((size_t)co * s->C_in + c) * KK, oh, ow, 0, &m, &t);
            if (do_max) base_op(s, x_c, w_max + ((size_t)co * s->C_in + c) * KK, oh, ow, 1, &M, &t);
            volatile float term;
            if (two) {
              volatile float pa = coef(alpha, s, c, co) * m;
              volatile float pb = coef(beta, s, c, co) * M;
              term = pa + pb;
            } else {
              term = do_min ? m : M;
            }
            acc = acc + term;
          }
          y[(((size_t)n * s->C_out + co) * Ho + oh) * Wo + ow] = acc;
        }
  return 0;
}

/*
 * Backward of the forward above, all gradients in one sweep (any output may be NULL).
 * grad_x [N, C_in, H, W]; grad_w_min / grad_w_max OIHW (single-branch layers: the live one;
 * compound: ONE tensor, grad_w_min if non-NULL else grad_w_max, receives both branches);
 * grad_alpha / grad_beta [C_in, C_out] (two-parameter layers only).  All double, overwritten.
 */
int oracle_tsum_backward(const oracle_shape* s, int mode, const float* x, const float* w_min,
                         const float* w_max, const float* alpha, const float* beta, const float* gy,
                         double* grad_x, double* grad_w_min, double* grad_w_max, double* grad_alpha,
                         double* grad_beta) {
  int32_t Ho, Wo;
  if (out_shape(s, &Ho, &Wo) != 0) return -1;
  const int do_min = (mode != ORACLE_MAX), do_max = (mode != ORACLE_MIN);
  const int two = (mode == ORACLE_COMPOUND || mode == ORACLE_PARALLEL);
  if (mode == ORACLE_COMPOUND) {
    w_min = w_max = (w_min ? w_min : w_max);
    grad_w_min = grad_w_max = (grad_w_min ? grad_w_min : grad_w_max);
  }
  if (!x || !gy || (do_min && !w_min) || (do_max && !w_max)) return -1;
  if (!two && (grad_alpha || grad_beta)) return -1;
  const size_t KK = (size_t)s->KH * s->KW, HW = (size_t)s->H * s->W;
  const size_t nw = (size_t)s->C_out * s->C_in * KK, nab = (size_t)s->C_in * s->C_out;
  if (grad_x) memset(grad_x, 0, sizeof(double) * s->N * s->C_in * HW);
  if (do_min && grad_w_min) memset(grad_w_min, 0, sizeof(double) * nw);
  if (do_max && grad_w_max) memset(grad_w_max, 0, sizeof(double) * nw);
  if (grad_alpha) memset(grad_alpha, 0, sizeof(double) * nab);
  if (grad_beta) memset(grad_beta, 0, sizeof(double) * nab);
  for (int n = 0; n < s->N; ++n)
    for (int co = 0; co < s->C_out; ++co)
      for (int oh = 0; oh < Ho; ++oh)
        for (int ow = 0; ow < Wo; ++ow) {
          const double g = gy[(((size_t)n * s->C_out + co) * Ho + oh) * Wo + ow];
          for (int c = 0; c < s->C_in; ++c) {
            const float* x_c = x + ((size_t)n * s->C_in + c) * HW;
            for (int br = 0; br < 2; ++br) { /* 0: min-plus branch, 1: max-plus branch */
              if ((br == 0 && !do_min) || (br == 1 && !do_max)) continue;
              const float* w_cc = (br ? w_max : w_min) + ((size_t)co * s->C_in + c) * KK;
              float v;
              int32_t t;
              base_op(s, x_c, w_cc, oh, ow, br, &v, &t);
              const double cf = two ? (double)coef(br ? beta : alpha, s, c, co) : 1.0;
              const int i = t / s->KW, j = t % s->KW;
              const int ih = oh * s->stride_h - s->pad_h + i * s->dil_h;
              const int iw = ow * s->stride_w - s->pad_w + j * s->dil_w;
              if (grad_x) grad_x[((size_t)n * s->C_in + c) * HW + (size_t)ih * s->W + iw] += cf * g;
              double* gw = br ? grad_w_max : grad_w_min;
              if (gw) gw[((size_t)co * s->C_in + c) * KK + t] += cf * g;
              double* gc = br ? grad_beta : grad_alpha;
              if (gc) gc[(size_t)c * s->C_out + co] += g * (double)v;
            }
          }
        }
  return 0;
}
