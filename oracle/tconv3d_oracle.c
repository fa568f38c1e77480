/*
 * CPU oracle for the three-dimensional tropical convolution layers.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow loop nest written from the
 * paper's definitions.  Only the tests, the smoke check and the benchmark's cpu_baseline leg may call
 * it.  It shares no code, header, table or helper with the HIP library.
 *
 * What it computes (paper Sec. 3.2, three-dimensional case).  Base operators for one input channel:
 *   MinPlus3d(X, W, h, w, d, c_in, c_out) = min over the KH x KW x KD window of X[h+i, w+j, d+a, c_in] + W[i, j, a, c_in, c_out],
 *   MaxPlus3d with max.  Layers (iii) - (vi) reduce the base operator over c_in with max or min, as in one and
 *   two dimensions; compound / parallel (Sec. 3.3): y = alpha[c_out]*y_min + beta[c_out]*y_max.
 *
 * Readings: tensors x [N, C_in, D, H, W], kernels [C_out, C_in, KD, KH, KW], outputs [N, C_out, D_out, H_out,
 * W_out] (depth is the slowest spatial axis, as volumetric tensors are usually stored); per axis
 * out = floor((in + 2*pad - dil*(k-1) - 1)/stride) + 1 and input position o*stride - pad + tap*dil; padding holds
 * the semiring identity (tap skipped; pad <= dil*(k-1) per axis); the saved winner is the flattened tap
 * k = ((c*KD + a)*KH + i)*KW + j; ties keep the lowest k (layers (iii), (vi): the lowest tap inside the lowest
 * channel); every x + w is one rounded fp32 add; y = fl(fl(alpha*y_min) + fl(beta*y_max)); backward sends the whole
 * gradient of a branch through its winner, scaled by alpha / beta in compound and parallel mode, sums in double.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct oracle3d_shape {
  int32_t N, C_in, D, H, W, C_out, KD, KH, KW;
  int32_t stride[3], pad[3], dil[3]; /* depth, height, width */
} oracle3d_shape;

enum { O_MAX = 0, O_MIN = 1, O_COMPOUND = 2, O_PARALLEL = 3, O_MINPLUS_MAX = 4, O_MAXPLUS_MIN = 5 };

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

static int out_dim(long in, long k, long stride, long pad, long dil, int32_t* out) {
  long ext = dil * (k - 1), n = in + 2 * pad - ext - 1;
  if (in < 1 || k < 1 || stride < 1 || dil < 1 || pad < 0 || n < 0 || pad > ext) return -1;
  *out = (int32_t)(n / stride + 1);
  return axis_has_empty_window(in, k, stride, pad, dil, *out) ? -1 : 0;
}

static int out_shape(const oracle3d_shape* s, int32_t* Do, int32_t* Ho, int32_t* Wo) {
  if (s->N < 1 || s->C_in < 1 || s->C_out < 1) return -1;
  return out_dim(s->D, s->KD, s->stride[0], s->pad[0], s->dil[0], Do) ||
         out_dim(s->H, s->KH, s->stride[1], s->pad[1], s->dil[1], Ho) ||
         out_dim(s->W, s->KW, s->stride[2], s->pad[2], s->dil[2], Wo);
}

/* Base operator of one channel at one output position: extremum over the valid taps and its lowest tap
 * t = (a*KH + i)*KW + j (-1 if the window lies wholly in the padding, which the pad limits exclude). */
static void base3d(const oracle3d_shape* s, const float* xc, const float* wc, int od, int oh, int ow, int want_max,
                   float* value, int* tap) {
  int found = 0;
  float best = 0.0f;
  *tap = -1;
  for (int a = 0; a < s->KD; ++a) {
    long id = (long)od * s->stride[0] - s->pad[0] + (long)a * s->dil[0];
    if (id < 0 || id >= s->D) continue;
    for (int i = 0; i < s->KH; ++i) {
      long ih = (long)oh * s->stride[1] - s->pad[1] + (long)i * s->dil[1];
      if (ih < 0 || ih >= s->H) continue;
      for (int j = 0; j < s->KW; ++j) {
        long iw = (long)ow * s->stride[2] - s->pad[2] + (long)j * s->dil[2];
        if (iw < 0 || iw >= s->W) continue;
        volatile float sum = xc[(id * s->H + ih) * s->W + iw] + wc[(a * s->KH + i) * s->KW + j];
        float v = sum;
        if (!found || (want_max ? (v > best) : (v < best))) {
          best = v;
          *tap = (a * s->KH + i) * s->KW + j;
          found = 1;
        }
      }
    }
  }
  *value = best;
}

static void branch(const oracle3d_shape* s, const float* xn, const float* wco, int od, int oh, int ow, int inner_max,
                   int outer_max, float* value, int32_t* k) {
  const long vol = (long)s->D * s->H * s->W;
  const int KK = s->KD * s->KH * s->KW;
  int found = 0;
  float best = 0.0f;
  for (int c = 0; c < s->C_in; ++c) {
    float v;
    int t = -1;
    base3d(s, xn + c * vol, wco + (long)c * KK, od, oh, ow, inner_max, &v, &t);
    if (t < 0) continue;
    if (!found || (outer_max ? (v > best) : (v < best))) {
      best = v;
      *k = c * KK + t;
      found = 1;
    }
  }
  *value = best;
}

int oracle_tconv3d_forward(const oracle3d_shape* s, int mode, const float* x, const float* w_min, const float* w_max,
                           const float* alpha, const float* beta, float* y, float* y_min, float* y_max,
                           int32_t* idx_min, int32_t* idx_max) {
  int32_t Do, Ho, Wo;
  if (out_shape(s, &Do, &Ho, &Wo) != 0 || !x || !y || mode < O_MAX || mode > O_MAXPLUS_MIN) return -1;
  const int do_min = (mode != O_MAX && mode != O_MAXPLUS_MIN), do_max = (mode != O_MIN && mode != O_MINPLUS_MAX);
  if (mode == O_COMPOUND) w_min = w_max = (w_min ? w_min : w_max);
  if ((do_min && (!w_min || !idx_min)) || (do_max && (!w_max || !idx_max))) return -1;
  const long vol = (long)s->D * s->H * s->W, ovol = (long)Do * Ho * Wo;
  const long K = (long)s->C_in * s->KD * s->KH * s->KW;
  const long planes = (long)s->N * s->C_out;
#pragma omp parallel for schedule(static)
  for (long pl = 0; pl < planes; ++pl) {
    const int n = (int)(pl / s->C_out), co = (int)(pl % s->C_out);
    const float* xn = x + (long)n * s->C_in * vol;
    for (int od = 0; od < Do; ++od)
      for (int oh = 0; oh < Ho; ++oh)
        for (int ow = 0; ow < Wo; ++ow) {
          const long o = pl * ovol + ((long)od * Ho + oh) * Wo + ow;
          float m = 0.0f, M = 0.0f, out;
          if (do_min) {
            branch(s, xn, w_min + co * K, od, oh, ow, 0, mode == O_MINPLUS_MAX, &m, &idx_min[o]);
            if (y_min) y_min[o] = m;
          }
          if (do_max) {
            branch(s, xn, w_max + co * K, od, oh, ow, 1, mode != O_MAXPLUS_MIN, &M, &idx_max[o]);
            if (y_max) y_max[o] = M;
          }
          if (!do_min) out = M;
          else if (!do_max) out = m;
          else {
            volatile float pa = (alpha ? alpha[co] : 1.0f) * m;
            volatile float pb = (beta ? beta[co] : 1.0f) * M;
            volatile float sum = pa + pb;
            out = sum;
          }
          y[o] = out;
        }
  }
  return 0;
}

int oracle_tconv3d_backward(const oracle3d_shape* s, int mode, const float* gy, const float* alpha, const float* beta,
                            const int32_t* idx_min, const int32_t* idx_max, double* grad_x, double* grad_w_min,
                            double* grad_w_max) {
  int32_t Do, Ho, Wo;
  if (out_shape(s, &Do, &Ho, &Wo) != 0 || !gy || mode < O_MAX || mode > O_MAXPLUS_MIN) return -1;
  const int do_min = (mode != O_MAX && mode != O_MAXPLUS_MIN), do_max = (mode != O_MIN && mode != O_MINPLUS_MAX);
  const int two = (mode == O_COMPOUND || mode == O_PARALLEL);
  if ((do_min && !idx_min) || (do_max && !idx_max)) return -1;
  if (mode == O_COMPOUND) grad_w_min = grad_w_max = (grad_w_min ? grad_w_min : grad_w_max);
  const long vol = (long)s->D * s->H * s->W;
  const int KK = s->KD * s->KH * s->KW;
  const long K = (long)s->C_in * KK;
  if (grad_x) memset(grad_x, 0, sizeof(double) * (size_t)s->N * s->C_in * vol);
  if (do_min && grad_w_min) memset(grad_w_min, 0, sizeof(double) * (size_t)s->C_out * K);
  if (do_max && grad_w_max && grad_w_max != grad_w_min) memset(grad_w_max, 0, sizeof(double) * (size_t)s->C_out * K);
  for (int n = 0; n < s->N; ++n)
    for (int co = 0; co < s->C_out; ++co)
      for (int od = 0; od < Do; ++od)
        for (int oh = 0; oh < Ho; ++oh)
          for (int ow = 0; ow < Wo; ++ow) {
            const long o = ((((long)n * s->C_out + co) * Do + od) * Ho + oh) * Wo + ow;
            const double g = (double)gy[o];
            for (int b = 0; b < 2; ++b) {
              if (b == 0 ? !do_min : !do_max) continue;
              const int32_t k = b == 0 ? idx_min[o] : idx_max[o];
              const double coef = !two ? 1.0 : (b == 0 ? (alpha ? (double)alpha[co] : 1.0) : (beta ? (double)beta[co] : 1.0));
              if (k < 0 || k >= K) return -2; /* not a winner index of this layer */
              const int c = k / KK, t = k % KK;
              const int a = t / (s->KH * s->KW), i = (t / s->KW) % s->KH, j = t % s->KW;
              const long id = (long)od * s->stride[0] - s->pad[0] + (long)a * s->dil[0];
              const long ih = (long)oh * s->stride[1] - s->pad[1] + (long)i * s->dil[1];
              const long iw = (long)ow * s->stride[2] - s->pad[2] + (long)j * s->dil[2];
              if (id < 0 || id >= s->D || ih < 0 || ih >= s->H || iw < 0 || iw >= s->W) return -2; /* a padded tap */
              if (grad_x) grad_x[((long)n * s->C_in + c) * vol + (id * s->H + ih) * s->W + iw] += coef * g;
              double* gw = b == 0 ? grad_w_min : grad_w_max;
              if (gw) gw[co * K + k] += coef * g;
            }
          }
  return 0;
}
