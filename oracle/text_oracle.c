/*
 * CPU oracle for the extensions of the tropical convolution layers: zero padding, the layer epilogue
 * (bias, folded batch-norm affine, residual add) and the half-precision arithmetic contract.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Plain, slow loops written from the paper; only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.  It shares no code, header,
 * table or helper with the HIP library, and none with the other oracle files either (its loop nest is
 * its own), so that it can be pinned AGAINST them.
 *
 * What it computes.
 *  - Operators: paper Sec. 3.1 (base operators, layers (iv) MinPlus-Min-Conv2d and (v) MaxPlus-Max-Conv2d)
 *    and Sec. 3.3 (compound, parallel), exactly as the main oracle reads them (NCHW / OIHW,
 *    cross-correlation, tap k = (c*KH + i)*KW + j, lowest k on ties, one rounded add per candidate,
 *    combine = two rounded products and a rounded sum).
 *  - Zero padding (App. A.1.1: the PyTorch formulation unfolds the input, and unfolding pads with
 *    zeros): with pad_zero != 0 an out-of-image tap is a candidate like any other, with input value +0,
 *    i.e. the sum fl(0 + w[k]); it can win, and then its index is saved like any other.  Backward: a
 *    winner that lies in the padding has no input element, so its gradient reaches the kernel only.
 *    With pad_zero == 0 out-of-image taps are skipped (the semiring identity of Sec. 3.1).
 *  - Epilogue (App. A.2: the layers derive from the framework's convolution base class, which carries
 *    an optional bias; Sec. 5, "TCNN BasicBlock": tropical conv -> batch norm -> tropical conv -> batch norm
 *    -> shortcut add, no activation): after the combine,
 *        t = y;  if bias: t = fl(t + bias[co]);  if scale: t = fl(fl(t * scale[co]) + shift[co]);
 *        if residual: t = fl(t + residual[n, co, oh, ow])
 *    every operation rounded to fp32 on its own.  scale / shift are a batch norm folded for inference
 *    (scale = gamma / sqrt(var + eps), shift = beta - mean * scale; forming them is the caller's business).
 *    The branch outputs y_min / y_max and the indices are those of the bare layer.
 *  - Half precision: x, the kernels and the outputs are IEEE binary16.  Every candidate is ONE add
 *    rounded to binary16 (round to nearest even), the comparison is on those binary16 sums, ties keep the
 *    lowest k.  The combine is evaluated in fp32 from the binary16 extrema (two rounded fp32 products, one
 *    rounded fp32 sum) and rounded to binary16 once.  (The paper trains in fp32; this is the contract of a
 *    packed 16-bit path, stated here.)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct text_shape {
  int32_t N, C_in, H, W;
  int32_t C_out, KH, KW;
  int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
} text_shape;

enum { TEXT_MAX = 0, TEXT_MIN = 1, TEXT_COMPOUND = 2, TEXT_PARALLEL = 3 };

/* 1 if some window of one axis has no tap inside the input (written out: every output position, every tap).  Under
 * identity padding the extremum of Sec. 3.1 over an empty set of taps is not defined, so such a layer is rejected. */
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

static int out_hw(const text_shape* s, int32_t* Ho, int32_t* Wo) {
  long nh = (long)s->H + 2L * s->pad_h - (long)s->dil_h * (s->KH - 1) - 1;
  long nw = (long)s->W + 2L * s->pad_w - (long)s->dil_w * (s->KW - 1) - 1;
  if (nh < 0 || nw < 0) return -1;
  *Ho = (int32_t)(nh / s->stride_h + 1);
  *Wo = (int32_t)(nw / s->stride_w + 1);
  return 0;
}

/* ---- binary16 <-> double, written out (no compiler half type involved) */
static double half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1, e = (h >> 10) & 31, m = h & 1023;
  double v;
  if (e == 0)
    v = ldexp((double)m, -24); /* subnormal: m * 2^-24 */
  else if (e == 31)
    v = m ? NAN : INFINITY;
  else
    v = ldexp((double)(1024 + m), e - 25); /* (1 + m/1024) * 2^(e-15) */
  return sign ? -v : v;
}

/* Round a double to the nearest binary16, ties to even; overflow gives infinity. */
static uint16_t double_to_half(double v) {
  uint16_t sign = (uint16_t)(signbit(v) ? 0x8000u : 0u);
  double a = fabs(v);
  if (isnan(v)) return (uint16_t)(sign | 0x7e00u);
  if (a == 0.0) return sign;
  if (isinf(v)) return (uint16_t)(sign | 0x7c00u);
  int ex;
  (void)frexp(a, &ex); /* a = f * 2^ex, f in [0.5, 1) : a in [2^(ex-1), 2^ex) */
  int e = ex - 1;      /* unbiased exponent of a */
  if (e < -14) e = -14; /* subnormal range: fixed quantum 2^-24 */
  /* quantum of the binary16 grid at this exponent: 2^(e-10) */
  double q = ldexp(1.0, e - 10);
  double n = a / q;          /* exact: a power-of-two scaling */
  double r = nearbyint(n);   /* current rounding mode is to-nearest-even */
  double res = r * q;
  if (res >= 65520.0) return (uint16_t)(sign | 0x7c00u); /* rounds past the largest finite value 65504 */
  /* re-encode */
  int ex2;
  (void)frexp(res, &ex2);
  int e2 = ex2 - 1;
  uint16_t bits;
  if (res < ldexp(1.0, -14)) {
    bits = (uint16_t)(res / ldexp(1.0, -24));
  } else {
    double frac = res / ldexp(1.0, e2) - 1.0; /* in [0, 1) */
    bits = (uint16_t)(((e2 + 15) << 10) | (int)(frac * 1024.0));
  }
  return (uint16_t)(sign | bits);
}

uint16_t text_double_to_half(double v) { return double_to_half(v); }
double text_half_to_double(uint16_t h) { return half_to_double(h); }

/* One output, one branch, fp32 arithmetic: taps in ascending k, strict compare. */
static void scan_f32(const text_shape* s, int pad_zero, const float* x_n, const float* w_co, int oh, int ow,
                     int want_max, float* best_out, int32_t* idx_out) {
  float best = 0.0f;
  int32_t bidx = -1;
  for (int c = 0; c < s->C_in; ++c)
    for (int i = 0; i < s->KH; ++i)
      for (int j = 0; j < s->KW; ++j) {
        int ih = oh * s->stride_h - s->pad_h + i * s->dil_h;
        int iw = ow * s->stride_w - s->pad_w + j * s->dil_w;
        int inside = (ih >= 0 && ih < s->H && iw >= 0 && iw < s->W);
        if (!inside && !pad_zero) continue;
        int32_t k = (c * s->KH + i) * s->KW + j;
        float xv = inside ? x_n[((size_t)c * s->H + ih) * s->W + iw] : 0.0f;
        volatile float sum = xv + w_co[k];
        float v = sum;
        if (bidx < 0 || (want_max ? (v > best) : (v < best))) {
          best = v;
          bidx = k;
        }
      }
  *best_out = best;
  *idx_out = bidx;
}

/*
 * Forward in fp32 with the padding mode and the epilogue.  Pointers that may be NULL: alpha, beta (ones),
 * bias, scale (then shift is ignored; with scale, a NULL shift means zeros), residual, y_min, y_max,
 * idx_min, idx_max (not written).  Returns 0, -1 on a bad shape or missing kernel.
 */
int text_forward(const text_shape* s, int mode, int pad_zero, const float* x, const float* w_min,
                 const float* w_max, const float* alpha, const float* beta, const float* bias,
                 const float* scale, const float* shift, const float* residual, float* y, float* y_min,
                 float* y_max, int32_t* idx_min, int32_t* idx_max) {
  int32_t Ho, Wo;
  if (out_hw(s, &Ho, &Wo) != 0 || Ho < 1 || Wo < 1) return -1;
  if (!pad_zero && (s->pad_h > s->dil_h * (s->KH - 1) || s->pad_w > s->dil_w * (s->KW - 1))) return -1;
  if (!pad_zero && (axis_has_empty_window(s->H, s->KH, s->stride_h, s->pad_h, s->dil_h, Ho) ||
                    axis_has_empty_window(s->W, s->KW, s->stride_w, s->pad_w, s->dil_w, Wo)))
    return -1;
  const int do_min = (mode != TEXT_MAX), do_max = (mode != TEXT_MIN);
  const float* wmn = w_min;
  const float* wmx = w_max;
  if (mode == TEXT_COMPOUND) wmn = wmx = (w_min ? w_min : w_max);
  if ((do_min && !wmn) || (do_max && !wmx)) return -1;
  const size_t K = (size_t)s->C_in * s->KH * s->KW, x_img = (size_t)s->C_in * s->H * s->W;
  for (int n = 0; n < s->N; ++n)
    for (int co = 0; co < s->C_out; ++co)
      for (int oh = 0; oh < Ho; ++oh)
        for (int ow = 0; ow < Wo; ++ow) {
          size_t o = (((size_t)n * s->C_out + co) * Ho + oh) * Wo + ow;
          float vmin = 0.0f, vmax = 0.0f;
          int32_t imin = -1, imax = -1;
          if (do_min) scan_f32(s, pad_zero, x + n * x_img, wmn + co * K, oh, ow, 0, &vmin, &imin);
          if (do_max) scan_f32(s, pad_zero, x + n * x_img, wmx + co * K, oh, ow, 1, &vmax, &imax);
          volatile float t;
          if (mode == TEXT_MAX)
            t = vmax;
          else if (mode == TEXT_MIN)
            t = vmin;
          else {
            volatile float pa = (alpha ? alpha[co] : 1.0f) * vmin;
            volatile float pb = (beta ? beta[co] : 1.0f) * vmax;
            t = pa + pb;
          }
          if (bias) t = t + bias[co];
          if (scale) {
            volatile float m = t * scale[co];
            t = m + (shift ? shift[co] : 0.0f);
          }
          if (residual) t = t + residual[o];
          if (y) y[o] = t;
          if (do_min && y_min) y_min[o] = vmin;
          if (do_max && y_max) y_max[o] = vmax;
          if (do_min && idx_min) idx_min[o] = imin;
          if (do_max && idx_max) idx_max[o] = imax;
        }
  return 0;
}

/*
 * Backward through saved winners that may lie in the (zero) padding: grad_w gets every winner's gradient,
 * grad_x only those whose tap is inside the image.  g_min = alpha*gy, g_max = beta*gy (compound / parallel),
 * g = gy (max / min).  Double sums, fixed order.  compound: both branches into grad_w_min if non-NULL else
 * grad_w_max.  Any of grad_x / grad_w_min / grad_w_max may be NULL (not computed).
 */
int text_backward(const text_shape* s, int mode, const float* gy, const float* alpha, const float* beta,
                  const int32_t* idx_min, const int32_t* idx_max, double* grad_x, double* grad_w_min,
                  double* grad_w_max) {
  int32_t Ho, Wo;
  if (out_hw(s, &Ho, &Wo) != 0) return -1;
  const int do_min = (mode != TEXT_MAX), do_max = (mode != TEXT_MIN);
  if ((do_min && !idx_min) || (do_max && !idx_max)) return -1;
  const size_t K = (size_t)s->C_in * s->KH * s->KW, x_img = (size_t)s->C_in * s->H * s->W;
  double* gmn = grad_w_min;
  double* gmx = grad_w_max;
  if (mode == TEXT_COMPOUND) gmn = gmx = (grad_w_min ? grad_w_min : grad_w_max);
  if (grad_x) memset(grad_x, 0, sizeof(double) * x_img * s->N);
  if (do_min && gmn) memset(gmn, 0, sizeof(double) * K * s->C_out);
  if (do_max && gmx) memset(gmx, 0, sizeof(double) * K * s->C_out);
  const int two = (mode == TEXT_COMPOUND || mode == TEXT_PARALLEL);
  for (int n = 0; n < s->N; ++n)
    for (int co = 0; co < s->C_out; ++co)
      for (int oh = 0; oh < Ho; ++oh)
        for (int ow = 0; ow < Wo; ++ow) {
          size_t o = (((size_t)n * s->C_out + co) * Ho + oh) * Wo + ow;
          for (int br = 0; br < 2; ++br) {
            if ((br == 0 && !do_min) || (br == 1 && !do_max)) continue;
            int32_t k = br ? idx_max[o] : idx_min[o];
            if (k < 0 || (size_t)k >= K) return -2;
            double coef = 1.0;
            if (two) coef = br ? (beta ? (double)beta[co] : 1.0) : (alpha ? (double)alpha[co] : 1.0);
            double g = coef * (double)gy[o];
            int j = k % s->KW, i = (k / s->KW) % s->KH, c = k / (s->KW * s->KH);
            int ih = oh * s->stride_h - s->pad_h + i * s->dil_h;
            int iw = ow * s->stride_w - s->pad_w + j * s->dil_w;
            if (grad_x && ih >= 0 && ih < s->H && iw >= 0 && iw < s->W)
              grad_x[n * x_img + ((size_t)c * s->H + ih) * s->W + iw] += g;
            double* gw = br ? gmx : gmn;
            if (gw) gw[(size_t)co * K + k] += g;
          }
        }
  return 0;
}

/* grad_bias[co] = sum over (n, oh, ow) of gy (the epilogue adds bias[co] to every output of the channel). */
int text_backward_bias(const text_shape* s, const float* gy, double* grad_bias) {
  int32_t Ho, Wo;
  if (out_hw(s, &Ho, &Wo) != 0) return -1;
  for (int co = 0; co < s->C_out; ++co) {
    double acc = 0.0;
    for (int n = 0; n < s->N; ++n)
      for (int q = 0; q < Ho * Wo; ++q) acc += (double)gy[((size_t)n * s->C_out + co) * Ho * Wo + q];
    grad_bias[co] = acc;
  }
  return 0;
}

/*
 * Half-precision forward (identity padding: out-of-image taps skipped, or zero padding).  x, kernels and the
 * outputs are binary16 bit patterns; alpha, beta fp32.  A candidate is the exact sum of its two binary16
 * operands (a double holds it exactly) rounded once to binary16; comparisons are on the rounded sums.
 */
int text_forward_f16(const text_shape* s, int mode, int pad_zero, const uint16_t* x, const uint16_t* w_min,
                     const uint16_t* w_max, const float* alpha, const float* beta, uint16_t* y,
                     uint16_t* y_min, uint16_t* y_max, int32_t* idx_min, int32_t* idx_max) {
  int32_t Ho, Wo;
  if (out_hw(s, &Ho, &Wo) != 0 || Ho < 1 || Wo < 1) return -1;
  if (!pad_zero && (s->pad_h > s->dil_h * (s->KH - 1) || s->pad_w > s->dil_w * (s->KW - 1))) return -1;
  if (!pad_zero && (axis_has_empty_window(s->H, s->KH, s->stride_h, s->pad_h, s->dil_h, Ho) ||
                    axis_has_empty_window(s->W, s->KW, s->stride_w, s->pad_w, s->dil_w, Wo)))
    return -1;
  const int do_min = (mode != TEXT_MAX), do_max = (mode != TEXT_MIN);
  const uint16_t* wk[2] = {w_min, w_max};
  if (mode == TEXT_COMPOUND) wk[0] = wk[1] = (w_min ? w_min : w_max);
  if ((do_min && !wk[0]) || (do_max && !wk[1])) return -1;
  const size_t K = (size_t)s->C_in * s->KH * s->KW, x_img = (size_t)s->C_in * s->H * s->W;
  for (int n = 0; n < s->N; ++n)
    for (int co = 0; co < s->C_out; ++co)
      for (int oh = 0; oh < Ho; ++oh)
        for (int ow = 0; ow < Wo; ++ow) {
          size_t o = (((size_t)n * s->C_out + co) * Ho + oh) * Wo + ow;
          double ext[2] = {0.0, 0.0}; /* the winning binary16 sums, as doubles */
          uint16_t ebits[2] = {0, 0};
          int32_t eidx[2] = {-1, -1};
          for (int br = 0; br < 2; ++br) {
            if ((br == 0 && !do_min) || (br == 1 && !do_max)) continue;
            for (int c = 0; c < s->C_in; ++c)
              for (int i = 0; i < s->KH; ++i)
                for (int j = 0; j < s->KW; ++j) {
                  int ih = oh * s->stride_h - s->pad_h + i * s->dil_h;
                  int iw = ow * s->stride_w - s->pad_w + j * s->dil_w;
                  int inside = (ih >= 0 && ih < s->H && iw >= 0 && iw < s->W);
                  if (!inside && !pad_zero) continue;
                  int32_t k = (c * s->KH + i) * s->KW + j;
                  double xv = inside ? half_to_double(x[n * x_img + ((size_t)c * s->H + ih) * s->W + iw]) : 0.0;
                  uint16_t hb = double_to_half(xv + half_to_double(wk[br][co * K + k]));
                  double hv = half_to_double(hb);
                  if (eidx[br] < 0 || (br ? (hv > ext[br]) : (hv < ext[br]))) {
                    ext[br] = hv;
                    ebits[br] = hb;
                    eidx[br] = k;
                  }
                }
          }
          uint16_t out;
          if (mode == TEXT_MAX)
            out = ebits[1];
          else if (mode == TEXT_MIN)
            out = ebits[0];
          else {
            volatile float pa = (alpha ? alpha[co] : 1.0f) * (float)ext[0];
            volatile float pb = (beta ? beta[co] : 1.0f) * (float)ext[1];
            volatile float sum = pa + pb;
            out = double_to_half((double)sum);
          }
          if (y) y[o] = out;
          if (do_min && y_min) y_min[o] = ebits[0];
          if (do_max && y_max) y_max[o] = ebits[1];
          if (do_min && idx_min) idx_min[o] = eidx[0];
          if (do_max && idx_max) idx_max[o] = eidx[1];
        }
  return 0;
}
