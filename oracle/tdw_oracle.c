/*
 * CPU oracle for the depthwise tropical convolution layer.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow loop nest written from the
 * paper's definitions.  Only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it.  It shares no code, header, table or helper with the HIP library.
 *
 * What it computes.  The MobileNetV2 variants of the paper (Sec. 5, deep-backbone experiments,
 * "MobileNetV2 Models") replace every depthwise convolution by a tropical layer with learnable alpha
 * and beta.  A depthwise layer gives every output channel ONE input channel, so the channel sum of
 * the Sum-channel layers (Sec. 3.1 (i), (ii); Sec. 3.5 / 3.6) has a single term and the layer is the
 * base operator of Sec. 3.1 applied per channel:
 *   m[n, co, oh, ow] = min over the KH x KW window of x[n, c, ih, iw] + w_min[co, i, j]       (MinPlus2d)
 *   M[n, co, oh, ow] = max over the window of            x[n, c, ih, iw] + w_max[co, i, j]       (MaxPlus2d)
 *   max layer: y = M;  min layer: y = m;
 *   compound: y = alpha[co]*m + beta[co]*M with w_min == w_max;  parallel: the same with two kernels.
 *
 * Readings where the paper is silent:
 *   - C_out = mult * C_in with an integer channel multiplier mult >= 1 (MobileNetV2: 1); output channel
 *     co reads input channel c = co / mult (the grouping of a depthwise convolution with groups = C_in);
 *     kernels are [C_out, 1, KH, KW], alpha and beta [C_out] (NULL = all ones; unused in max / min layers);
 *   - padding holds the semiring identity: a padded tap is skipped (pad <= dil*(k-1), so every window keeps
 *     a valid tap); ties keep the lowest tap t = i*KW + j (strict compare while t ascends);
 *   - every x + w is one rounded fp32 add; y = fl(fl(alpha*m) + fl(beta*M)), no fused multiply-add;
 *   - backward is the sub-gradient through the winner of each window, with g = gy[n, co, oh, ow]:
 *       grad_x[n, c, ih*, iw*] += alpha*g (min winner), += beta*g (max winner)   (g itself in max / min layers)
 *       grad_w_min[co, t*] += alpha*g, grad_w_max[co, t*] += beta*g (compound: both into ONE tensor)
 *       grad_alpha[co] += g*m, grad_beta[co] += g*M
 *     accumulated in double.
 */
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
  if (s->C_in < 1 || s->C_out < s->C_in || s->C_out % s->C_in != 0) return -1;
  *H_out = (int32_t)(nh / s->stride_h + 1);
  *W_out = (int32_t)(nw / s->stride_w + 1);
  if (axis_has_empty_window(s->H, s->KH, s->stride_h, s->pad_h, s->dil_h, *H_out) ||
      axis_has_empty_window(s->W, s->KW, s->stride_w, s->pad_w, s->dil_w, *W_out))
    return -1;
  return 0;
}

/* Base operator of Sec. 3.1 on one window of one channel plane: extremum of x + w over the valid taps,
 * its lowest tap and that tap's input offset inside the plane. */
static void window(const oracle_shape* s, const float* plane, const float* w, int oh, int ow, int want_max,
                   float* value, int* tap, long* x_off) {
  int found = 0;
  float best = 0.0f;
  for (int i = 0; i < s->KH; ++i) {
    int ih = oh * s->stride_h - s->pad_h + i * s->dil_h;
    if (ih < 0 || ih >= s->H) continue;
    for (int j = 0; j < s->KW; ++j) {
      int iw = ow * s->stride_w - s->pad_w + j * s->dil_w;
      if (iw < 0 || iw >= s->W) continue;
      volatile float sum = plane[(long)ih * s->W + iw] + w[i * s->KW + j];
      float v = sum;
      if (!found || (want_max ? (v > best) : (v < best))) {
        best = v;
        found = 1;
        *tap = i * s->KW + j;
        *x_off = (long)ih * s->W + iw;
      }
    }
  }
  *value = best;
}

/* tap_min / tap_max (optional, int32 per output): the winning tap t = i*KW + j of each live branch. */
int oracle_tdw_forward(const oracle_shape* s, int mode, const float* x, const float* w_min, const float* w_max,
                       const float* alpha, const float* beta, float* y, int32_t* tap_min, int32_t* tap_max) {
  int32_t Ho, Wo;
  if (out_shape(s, &Ho, &Wo) != 0 || !x || !y) return -1;
  const int do_min = (mode != ORACLE_MAX), do_max = (mode != ORACLE_MIN);
  if (mode == ORACLE_COMPOUND) w_min = w_max = (w_min ? w_min : w_max);
  if ((do_min && !w_min) || (do_max && !w_max)) return -1;
  const int mult = s->C_out / s->C_in, KK = s->KH * s->KW;
  const long planes = (long)s->N * s->C_out;
#pragma omp parallel for schedule(static)
  for (long pl = 0; pl < planes; ++pl) {
    const int n = (int)(pl / s->C_out), co = (int)(pl % s->C_out), c = co / mult;
    const float* plane = x + ((long)n * s->C_in + c) * s->H * s->W;
    for (int oh = 0; oh < Ho; ++oh)
      for (int ow = 0; ow < Wo; ++ow) {
        float m = 0.0f, M = 0.0f, out;
        int t_min = 0, t_max = 0;
        long off;
        if (do_min) window(s, plane, w_min + (long)co * KK, oh, ow, 0, &m, &t_min, &off);
        if (do_max) window(s, plane, w_max + (long)co * KK, oh, ow, 1, &M, &t_max, &off);
        if (mode == ORACLE_MAX) out = M;
        else if (mode == ORACLE_MIN) out = m;
        else {
          volatile float pa = (alpha ? alpha[co] : 1.0f) * m;
          volatile float pb = (beta ? beta[co] : 1.0f) * M;
          volatile float sum = pa + pb;
          out = sum;
        }
        y[(pl * Ho + oh) * Wo + ow] = out;
        if (do_min && tap_min) tap_min[(pl * Ho + oh) * Wo + ow] = t_min;
        if (do_max && tap_max) tap_max[(pl * Ho + oh) * Wo + ow] = t_max;
      }
  }
  return 0;
}

/* Any gradient pointer may be NULL (not wanted).  grad_w_min / grad_w_max: [C_out, KH*KW]; compound adds
 * both branches into grad_w_min (or grad_w_max if only that one is given). */
int oracle_tdw_backward(const oracle_shape* s, int mode, const float* x, const float* w_min, const float* w_max,
                        const float* alpha, const float* beta, const float* gy, double* grad_x,
                        double* grad_w_min, double* grad_w_max, double* grad_alpha, double* grad_beta) {
  int32_t Ho, Wo;
  if (out_shape(s, &Ho, &Wo) != 0 || !x || !gy) return -1;
  const int do_min = (mode != ORACLE_MAX), do_max = (mode != ORACLE_MIN);
  const int two = (mode == ORACLE_COMPOUND || mode == ORACLE_PARALLEL);
  if (mode == ORACLE_COMPOUND) {
    w_min = w_max = (w_min ? w_min : w_max);
    grad_w_min = grad_w_max = (grad_w_min ? grad_w_min : grad_w_max);
  }
  if ((do_min && !w_min) || (do_max && !w_max)) return -1;
  if (!two && (grad_alpha || grad_beta)) return -1;
  const int mult = s->C_out / s->C_in, KK = s->KH * s->KW;
  const long HW = (long)s->H * s->W;
  if (grad_x) memset(grad_x, 0, sizeof(double) * (size_t)s->N * s->C_in * HW);
  if (do_min && grad_w_min) memset(grad_w_min, 0, sizeof(double) * (size_t)s->C_out * KK);
  if (do_max && grad_w_max && grad_w_max != grad_w_min) memset(grad_w_max, 0, sizeof(double) * (size_t)s->C_out * KK);
  if (grad_alpha) memset(grad_alpha, 0, sizeof(double) * (size_t)s->C_out);
  if (grad_beta) memset(grad_beta, 0, sizeof(double) * (size_t)s->C_out);
  /* everything an input channel touches (its plane of grad_x, the kernels and coefficients of its output
   * channels) belongs to that channel alone, so channels can run side by side */
#pragma omp parallel for schedule(dynamic, 1)
  for (int c = 0; c < s->C_in; ++c)
    for (int n = 0; n < s->N; ++n) {
      const float* plane = x + ((long)n * s->C_in + c) * HW;
      double* gplane = grad_x ? grad_x + ((long)n * s->C_in + c) * HW : NULL;
      for (int co = c * mult; co < (c + 1) * mult; ++co) {
        const double a = (two && alpha) ? (double)alpha[co] : 1.0, b = (two && beta) ? (double)beta[co] : 1.0;
        for (int oh = 0; oh < Ho; ++oh)
          for (int ow = 0; ow < Wo; ++ow) {
            const double g = (double)gy[(((long)n * s->C_out + co) * Ho + oh) * Wo + ow];
            float v;
            int t;
            long off;
            if (do_min) {
              window(s, plane, w_min + (long)co * KK, oh, ow, 0, &v, &t, &off);
              if (gplane) gplane[off] += a * g;
              if (grad_w_min) grad_w_min[(long)co * KK + t] += a * g;
              if (grad_alpha) grad_alpha[co] += g * (double)v;
            }
            if (do_max) {
              window(s, plane, w_max + (long)co * KK, oh, ow, 1, &v, &t, &off);
              if (gplane) gplane[off] += b * g;
              if (grad_w_max) grad_w_max[(long)co * KK + t] += b * g;
              if (grad_beta) grad_beta[co] += g * (double)v;
            }
          }
      }
    }
  return 0;
}
