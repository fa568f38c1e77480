/*
 * CPU oracle for the one-dimensional tropical convolution layers.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow loop nest written from the
 * paper's definitions.  Only the tests, the smoke check and the benchmark's cpu_baseline leg may call
 * it.  It shares no code, header, table or helper with the HIP library.
 *
 * What it computes (paper Sec. 3.2, one-dimensional case).  Base operators for one input channel:
 *   MinPlus1d(X, W, l, c_in, c_out) = min over i in [K] of X[l + i, c_in] + W[i, c_in, c_out],  MaxPlus1d with max.
 * Layers: (iv) MinPlus-Min-Conv1d = min over c_in of MinPlus1d, (v) MaxPlus-Max-Conv1d = max over c_in of
 * MaxPlus1d, (iii) MinPlus-Max-Conv1d = max over c_in of MinPlus1d, (vi) MaxPlus-Min-Conv1d = min over c_in
 * of MaxPlus1d; compound / parallel (Sec. 3.3): y = alpha[c_out]*y_min + beta[c_out]*y_max over the layers
 * (iv) and (v), with one shared kernel (compound) or two (parallel).
 *
 * Readings, the same as for the two-dimensional layers: tensors x [N, C_in, L], kernels [C_out, C_in, K],
 * outputs [N, C_out, L_out], L_out = floor((L + 2*pad - dil*(K-1) - 1)/stride) + 1, input position
 * l*stride - pad + i*dil; padding holds the semiring identity (tap skipped; pad <= dil*(K-1)); the saved
 * winner is the flattened tap k = c*K + i; ties keep the lowest k (layers (iii), (vi): the lowest tap inside
 * the lowest channel); every x + w is one rounded fp32 add; y = fl(fl(alpha*y_min) + fl(beta*y_max));
 * backward sends the whole gradient of a branch through its winner, scaled by alpha / beta in compound and
 * parallel mode, sums in double.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct oracle1d_shape {
  int32_t N, C_in, L, C_out, K, stride, pad, dil;
} oracle1d_shape;

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

static int out_len(const oracle1d_shape* s, int32_t* L_out) {
  long ext = (long)s->dil * (s->K - 1);
  long n = (long)s->L + 2L * s->pad - ext - 1;
  if (s->N < 1 || s->C_in < 1 || s->L < 1 || s->C_out < 1 || s->K < 1 || s->stride < 1 || s->dil < 1 || s->pad < 0) return -1;
  if (n < 0 || s->pad > ext) return -1;
  *L_out = (int32_t)(n / s->stride + 1);
  return axis_has_empty_window(s->L, s->K, s->stride, s->pad, s->dil, *L_out) ? -1 : 0;
}

/* Base operator of one channel at output position l: extremum over the valid taps and its lowest tap. */
static void base1d(const oracle1d_shape* s, const float* xc, const float* wc, int l, int want_max, float* value,
                   int* tap) {
  int found = 0;
  float best = 0.0f;
  *tap = -1; /* stays -1 if this channel's window lies wholly in the padding */
  for (int i = 0; i < s->K; ++i) {
    long pos = (long)l * s->stride - s->pad + (long)i * s->dil;
    if (pos < 0 || pos >= s->L) continue;
    volatile float sum = xc[pos] + wc[i];
    float v = sum;
    if (!found || (want_max ? (v > best) : (v < best))) {
      best = v;
      *tap = i;
      found = 1;
    }
  }
  *value = best;
}

/* One branch of one output: the inner operator (inner_max) per channel, the outer one (outer_max) over the
 * channels in ascending order with a strict compare. */
static void branch(const oracle1d_shape* s, const float* xn, const float* wco, int l, int inner_max, int outer_max,
                   float* value, int32_t* k) {
  int found = 0;
  float best = 0.0f;
  for (int c = 0; c < s->C_in; ++c) {
    float v;
    int t = -1;
    base1d(s, xn + (long)c * s->L, wco + (long)c * s->K, l, inner_max, &v, &t);
    if (t < 0) continue;
    if (!found || (outer_max ? (v > best) : (v < best))) {
      best = v;
      *k = c * s->K + t;
      found = 1;
    }
  }
  *value = best;
}

int oracle_tconv1d_forward(const oracle1d_shape* s, int mode, const float* x, const float* w_min, const float* w_max,
                           const float* alpha, const float* beta, float* y, float* y_min, float* y_max,
                           int32_t* idx_min, int32_t* idx_max) {
  int32_t Lo;
  if (out_len(s, &Lo) != 0 || !x || !y || mode < O_MAX || mode > O_MAXPLUS_MIN) return -1;
  const int do_min = (mode != O_MAX && mode != O_MAXPLUS_MIN), do_max = (mode != O_MIN && mode != O_MINPLUS_MAX);
  if (mode == O_COMPOUND) w_min = w_max = (w_min ? w_min : w_max);
  if ((do_min && (!w_min || !idx_min)) || (do_max && (!w_max || !idx_max))) return -1;
  const long planes = (long)s->N * s->C_out;
#pragma omp parallel for schedule(static)
  for (long pl = 0; pl < planes; ++pl) {
    const int n = (int)(pl / s->C_out), co = (int)(pl % s->C_out);
    const float* xn = x + (long)n * s->C_in * s->L;
    for (int l = 0; l < Lo; ++l) {
      const long o = pl * Lo + l;
      float m = 0.0f, M = 0.0f, out;
      if (do_min) { /* min side: layer (iv), or (iii) = max over channels of the min-plus operator */
        branch(s, xn, w_min + (long)co * s->C_in * s->K, l, 0, mode == O_MINPLUS_MAX, &m, &idx_min[o]);
        if (y_min) y_min[o] = m;
      }
      if (do_max) {
        branch(s, xn, w_max + (long)co * s->C_in * s->K, l, 1, mode != O_MAXPLUS_MIN, &M, &idx_max[o]);
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

/* grad_x [N, C_in, L] and grad_w_min / grad_w_max [C_out, C_in, K] in double (any may be NULL); compound adds
 * both branches into grad_w_min (or grad_w_max if only that one is given). */
int oracle_tconv1d_backward(const oracle1d_shape* s, int mode, const float* gy, const float* alpha, const float* beta,
                            const int32_t* idx_min, const int32_t* idx_max, double* grad_x, double* grad_w_min,
                            double* grad_w_max) {
  int32_t Lo;
  if (out_len(s, &Lo) != 0 || !gy || mode < O_MAX || mode > O_MAXPLUS_MIN) return -1;
  const int do_min = (mode != O_MAX && mode != O_MAXPLUS_MIN), do_max = (mode != O_MIN && mode != O_MINPLUS_MAX);
  const int two = (mode == O_COMPOUND || mode == O_PARALLEL);
  if ((do_min && !idx_min) || (do_max && !idx_max)) return -1;
  if (mode == O_COMPOUND) grad_w_min = grad_w_max = (grad_w_min ? grad_w_min : grad_w_max);
  const long KW = (long)s->C_in * s->K;
  if (grad_x) memset(grad_x, 0, sizeof(double) * (size_t)s->N * s->C_in * s->L);
  if (do_min && grad_w_min) memset(grad_w_min, 0, sizeof(double) * (size_t)s->C_out * KW);
  if (do_max && grad_w_max && grad_w_max != grad_w_min) memset(grad_w_max, 0, sizeof(double) * (size_t)s->C_out * KW);
  for (int n = 0; n < s->N; ++n)
    for (int co = 0; co < s->C_out; ++co)
      for (int l = 0; l < Lo; ++l) {
        const long o = ((long)n * s->C_out + co) * Lo + l;
        const double g = (double)gy[o];
        for (int b = 0; b < 2; ++b) {
          if (b == 0 ? !do_min : !do_max) continue;
          const int32_t k = b == 0 ? idx_min[o] : idx_max[o];
          const double coef = !two ? 1.0 : (b == 0 ? (alpha ? (double)alpha[co] : 1.0) : (beta ? (double)beta[co] : 1.0));
          if (k < 0 || k >= KW) return -2; /* not a winner index of this layer */
          const int c = k / s->K, i = k % s->K;
          const long pos = (long)l * s->stride - s->pad + (long)i * s->dil;
          if (pos < 0 || pos >= s->L) return -2; /* a padded tap */
          if (grad_x) grad_x[((long)n * s->C_in + c) * s->L + pos] += coef * g;
          double* gw = b == 0 ? grad_w_min : grad_w_max;
          if (gw) gw[(long)co * KW + k] += coef * g;
        }
      }
  return 0;
}
